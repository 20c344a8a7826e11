// Attention kernels for gfx950: over the compacted cache (Sec. 3 first paragraph: the kept tokens are what
// later tokens attend to; every cached row is visible, the cache holds earlier blocks only) and, behind the
// cache rows, over the current block's own keys under the causal mask (the block's prefill attention, whose
// log-sum-exp of the window rows is the complete statistic of Sec. 3.3 "Precision").
//
//   attend_kernel          few query rows (decoding).  Workgroup = (key split, group of 256 query rows, KV
//                          head); the waves share row tiles over different key tiles.  The split's keys and
//                          values pass through LDS in chunks; each wave keeps 32 query rows in registers and an
//                          online-softmax state (reference, sum, unnormalised output) per row; the waves'
//                          states meet in LDS and leave one partial per split                          [MFMA]
//   attend_rows_kernel     a row tile per wave (window rows, whole blocks): two LDS stages, the next tile's
//                          logits issued before the current tile's softmax; writes the result itself when a
//                          workgroup sees all keys of its rows                                         [MFMA]
//   attend_combine_kernel  merges the partials of a row through their references and writes the output and
//                          the natural-log normaliser, the number laserkv_set_row_lse takes
//   attend_lse_kernel (+ attend_lse_combine_kernel)  the normaliser alone, for callers that want nothing else
#include "laserkv_device.h"
#include "laserkv_kernels.h"

namespace lkv {

constexpr int ATT_WAVES = 8;
constexpr int ATT_THREADS = ATT_WAVES * 64;
constexpr int ATT_ROWS = 256;      // query rows per workgroup: up to 8 row tiles
constexpr int ATT_MAX_SPLITS = 64;

// Keys per LDS chunk of attend_kernel (as many as its prefetch registers hold).
template <int DT>
__host__ __device__ constexpr int att_chunk_keys() { return DT == DT_BF16 ? 256 : 128; }

// Transposes, inside groups of 8 consecutive lanes, the 8 x 8 matrix of 16-bit elements whose row i is lane
// i's 16 bytes: afterwards lane i holds column i, element e of it being what lane e held at position i.
// Three exchange steps, each swapping one bit of the lane index with one bit of the element index; lane
// exchanges are DPP moves and every step is a select (no branches, no LDS traffic).
__device__ __forceinline__ uint4 transpose_8x8_b16(const uint4& v, int lane) {
  uint32_t x[4] = {v.x, v.y, v.z, v.w};
  const bool i0 = lane & 1, i1 = lane & 2, i2 = lane & 4;
  // lane bit 0 <-> half of the word: an even lane keeps its low half and takes the partner's low half as its
  // high half; an odd lane takes the partner's high half as its low half and keeps its high half
  const uint32_t sel = i0 ? 0x03020706u : 0x05040100u;  // byte picks from {partner (bytes 4-7), own (bytes 0-3)}
#pragma unroll
  for (int w = 0; w < 4; ++w) x[w] = __builtin_amdgcn_perm(lane_xor1(x[w]), x[w], sel);
#pragma unroll
  for (int a = 0; a < 4; a += 2) {  // lane bit 1 <-> word bit 0
    const uint32_t recv = lane_xor2(i1 ? x[a] : x[a + 1]);
    x[a] = i1 ? recv : x[a];
    x[a + 1] = i1 ? x[a + 1] : recv;
  }
#pragma unroll
  for (int a = 0; a < 2; ++a) {  // lane bit 2 <-> word bit 1
    const uint32_t recv = lane_xor4(i2 ? x[a] : x[a + 2], i2);
    x[a] = i2 ? recv : x[a];
    x[a + 2] = i2 ? x[a + 2] : recv;
  }
  return make_uint4(x[0], x[1], x[2], x[3]);
}

// The same for 4 x 4 matrices of 32-bit elements inside groups of 4 consecutive lanes.
__device__ __forceinline__ uint4 transpose_4x4_b32(const uint4& v, int lane) {
  uint32_t x[4] = {v.x, v.y, v.z, v.w};
  const bool i0 = lane & 1, i1 = lane & 2;
#pragma unroll
  for (int a = 0; a < 4; a += 2) {
    const uint32_t recv = lane_xor1(i0 ? x[a] : x[a + 1]);
    x[a] = i0 ? recv : x[a];
    x[a + 1] = i0 ? x[a + 1] : recv;
  }
#pragma unroll
  for (int a = 0; a < 2; ++a) {
    const uint32_t recv = lane_xor2(i1 ? x[a] : x[a + 2]);
    x[a] = i1 ? recv : x[a];
    x[a + 2] = i1 ? x[a + 2] : recv;
  }
  return make_uint4(x[0], x[1], x[2], x[3]);
}

// Writes one transposed group (the group's EPC consecutive keys at one head-dimension index) into that index's
// row of V^T.  fp32: keys in order.  bf16: the P operand of O^T += V^T P^T holds, per lane half kg and 16-key
// block, keys 4kg + (0..3) and 8 + 4kg + (0..3) (the accumulator layout of S^T); the row stores every 16-key
// block in that order, [0-3, 8-11 | 4-7, 12-15], so that a lane's eight keys are one 16-byte read.
template <int DT>
__device__ __forceinline__ void store_vt(uint4* row, int group, const uint4& t) {
  if (DT == DT_BF16) {
    uint2* r2 = reinterpret_cast<uint2*>(row) + 4 * (group >> 1) + (group & 1);
    r2[0] = make_uint2(t.x, t.y);
    r2[2] = make_uint2(t.z, t.w);
  } else {
    row[group] = t;
  }
}

// ds_read_b64_tr_b16: four 16-bit values per lane, transposed within groups of 16 lanes (see its use)
typedef short s16x4_lds __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint2 ds_read_tr16(const void* lds_ptr) {
  const s16x4_lds v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_lds*)lds_ptr);
  return __builtin_bit_cast(uint2, v);
}

// Workgroup barrier for data exchanged through LDS only: waits for this wave's LDS traffic, not for its
// global loads, so the next chunk's prefetch stays in flight across it (__syncthreads would wait for it).
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 t = {(__bf16)lo, (__bf16)hi};  // round to nearest even
  return __builtin_bit_cast(uint32_t, t);
}

// One pass over the split's keys for launches with few query rows (the waves of a workgroup share row tiles
// over different key tiles): its share of the cache rows, then its share of the block's own keys (none
// for attention over the cache alone).  S^T = K Q^T puts a query row in a lane (column rl of the tile; the two
// halves kg of the wave hold the same rows over different keys), so the softmax state is lane-private, and
// the 16 accumulator registers are already the B operand of O^T += V^T P^T: register r of half kg is key
// acc_row(r, kg), so a group of 8 (bf16) or 4 (f32) registers is one 16-byte operand chunk whose keys the A
// operand matches by reading V^T at the same key offsets.  V is transposed in registers on its way into LDS.
// Block key i is visible to query j iff i <= diag + j: chunks past the last row of the workgroup are never
// loaded, tiles past the last row of the wave are skipped, tiles that cross a row's limit take a masked path.
template <int DT, int D, int KC>
__global__ __launch_bounds__(ATT_THREADS) void attend_kernel(AttendParams p) {
  constexpr int ES = DT == DT_BF16 ? 2 : 4;
  constexpr int CH = D * ES / 16;             // 16-byte chunks per row
  constexpr int NCH = CH / 2;
  constexpr int CHP = CH + 1;                 // K row pitch in chunks (odd)
  constexpr int EPC = 16 / ES;                // elements per 16-byte chunk
  constexpr int VTP = KC / EPC + 1;           // V^T row pitch in chunks (odd)
  constexpr int KL = KC * CH / ATT_THREADS;   // 16-byte loads per thread, tensor and chunk
  constexpr int NDT = D / 32;                 // 32-wide tiles of the head dimension
  constexpr int TPC = KC / 32;                // key tiles per chunk
  constexpr int RUNS = 32 / (2 * EPC);        // operand chunks per lane and 32-key tile in P.V
  constexpr int K_ROWS_PER_LOAD = ATT_THREADS / CH;
  constexpr int V_GROUPS_PER_LOAD = ATT_THREADS / (EPC * CH);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, rl = lane & 31, kg = lane >> 5;
  // consecutive indices stay on one XCD: the row groups and splits of a head share that XCD's L2
  const int n_wg = gridDim.x;
  const int idx = xcd_major(blockIdx.x, n_wg);
  const int split = idx % p.n_splits, qg = (idx / p.n_splits) % p.n_qgroups, h = idx / (p.n_splits * p.n_qgroups);
  const int wprt = 1 << p.wprt_log;           // waves that share a row tile, over different key tiles
  const int rt = wave >> p.wprt_log, ks = wave & (wprt - 1);
  const int row = qg * ATT_ROWS + rt * 32 + rl;

  extern __shared__ uint4 smem[];
  uint4* sK = smem;                           // [KC][CHP]
  uint4* sVT = smem + KC * CHP;               // [D][VTP]: V^T, element (d, key) at chunk key / EPC of row d

  // the wave's 32 query rows, as the B operand of S^T
  uint4 a[NCH];
  int blk_end_lane;  // block keys [0, blk_end_lane) are visible to this lane's row
  {
    const int m = min(row, p.m_rows - 1);
    const int g = m / p.n_q, j = m - g * p.n_q;
    const char* ptr = p.q.base + (int64_t)(h * p.group + g) * p.q.stride_head + (int64_t)j * p.q.stride_row;
#pragma unroll
    for (int i = 0; i < NCH; ++i) a[i] = ld16(ptr + (2 * i + kg) * 16);
    blk_end_lane = max(0, min(p.s_t, p.diag + j + 1));
  }
  // key ranges of this split in the two segments; the block range ends where the last row of the workgroup
  // stops seeing keys
  const int lo0 = min(split * p.keys_per_split, p.cache_len), hi0 = min(lo0 + p.keys_per_split, p.cache_len);
  int lo1 = 0, hi1 = 0;
  if (p.s_t > 0) {
    const int m0 = qg * ATT_ROWS, m1 = min(m0 + ATT_ROWS, p.m_rows) - 1;
    const int g0 = m0 / p.n_q, g1 = m1 / p.n_q;
    const int j_max = g0 == g1 ? m1 - g1 * p.n_q : p.n_q - 1;
    const int wg_end = max(0, min(p.s_t, p.diag + j_max + 1));
    lo1 = min(split * p.blk_keys_per_split, wg_end);
    hi1 = min(lo1 + p.blk_keys_per_split, wg_end);
  }

  const __amdgpu_buffer_rsrc_t ksrd0 = make_srd(p.k_cache + (int64_t)h * p.cache_stride_head, (uint32_t)p.cache_len * (uint32_t)p.row_bytes);
  const __amdgpu_buffer_rsrc_t vsrd0 = make_srd(p.v_cache + (int64_t)h * p.cache_stride_head, (uint32_t)p.cache_len * (uint32_t)p.row_bytes);
  const uint32_t kb_bytes = p.s_t > 0 ? (uint32_t)(p.s_t - 1) * (uint32_t)p.kb_stride_row + (uint32_t)p.row_bytes : 0u;
  const uint32_t vb_bytes = p.s_t > 0 ? (uint32_t)(p.s_t - 1) * (uint32_t)p.vb_stride_row + (uint32_t)p.row_bytes : 0u;
  const __amdgpu_buffer_rsrc_t ksrd1 = make_srd(p.k_blk + (int64_t)h * p.kb_stride_head, kb_bytes);
  const __amdgpu_buffer_rsrc_t vsrd1 = make_srd(p.v_blk + (int64_t)h * p.vb_stride_head, vb_bytes);
  // K: chunk tid % CH of row tid / CH (+ K_ROWS_PER_LOAD per load).  V: lane groups of EPC consecutive lanes
  // hold EPC consecutive keys at the same chunk, the shape the register transpose wants.
  const uint32_t k_row = tid / CH, k_col = tid % CH;
  const uint32_t v_i = tid % EPC, v_c = (tid / EPC) % CH, v_grp = tid / (EPC * CH);
  uint4 kpre[KL], vpre[KL];
  auto prefetch = [&](int seg, int kc0) {
    const __amdgpu_buffer_rsrc_t ksrd = seg ? ksrd1 : ksrd0, vsrd = seg ? vsrd1 : vsrd0;
    const uint32_t kstride = seg ? (uint32_t)p.kb_stride_row : (uint32_t)p.row_bytes;
    const uint32_t vstride = seg ? (uint32_t)p.vb_stride_row : (uint32_t)p.row_bytes;
#pragma unroll
    for (int u = 0; u < KL; ++u) {
      kpre[u] = buf_ld16(ksrd, (uint32_t)(kc0 + k_row + u * K_ROWS_PER_LOAD) * kstride + k_col * 16);
      const uint32_t key = (u * V_GROUPS_PER_LOAD + v_grp) * EPC + v_i;
      vpre[u] = buf_ld16(vsrd, (uint32_t)(kc0 + key) * vstride + v_c * 16);
    }
  };

  float m_ref = NEG_BIG, l_sum = 0.0f;
  f32x16 o[NDT];
#pragma unroll
  for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.0f;

  int seg = lo0 < hi0 ? 0 : 1;
  int kc0 = seg ? lo1 : lo0;
  bool have = seg ? lo1 < hi1 : true;
  if (have) prefetch(seg, kc0);
  while (have) {
    lds_barrier();  // every wave has finished with the previous chunk
#pragma unroll
    for (int u = 0; u < KL; ++u) {
      sK[(k_row + u * K_ROWS_PER_LOAD) * CHP + k_col] = kpre[u];
      const uint4 t = DT == DT_BF16 ? transpose_8x8_b16(vpre[u], lane) : transpose_4x4_b32(vpre[u], lane);
      // the lane now holds head-dimension index v_c * EPC + v_i for the group's EPC keys
      store_vt<DT>(sVT + (v_c * EPC + v_i) * VTP, u * V_GROUPS_PER_LOAD + v_grp, t);
    }
    // the chunk after this one: the next of the segment, else the first of the block's keys
    int nseg = seg, nkc = kc0 + KC;
    bool nhave = nkc < (seg ? hi1 : hi0);
    if (!nhave && seg == 0 && lo1 < hi1) {
      nseg = 1;
      nkc = lo1;
      nhave = true;
    }
    if (nhave) prefetch(nseg, nkc);  // in flight while this chunk is worked on
    lds_barrier();

    const int k_hi = seg ? hi1 : hi0;
    const int lane_end = seg ? min(hi1, blk_end_lane) : hi0;  // end of the keys of this segment the lane's row sees
#pragma unroll 1
    for (int nt = ks; nt < TPC; nt += wprt) {
      const int kbase = kc0 + nt * 32;
      if (kbase >= k_hi) break;  // wave-uniform
      const int n_vis = lane_end - kbase;  // keys of this tile the lane's row sees (>= 32: all)
      if (!__any(n_vis > 0)) continue;     // the tile lies past the limit of every row of the wave
      f32x16 acc;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
      const uint4* krow = sK + (size_t)(nt * 32 + rl) * CHP + kg;
#pragma unroll
      for (int i = 0; i < NCH; ++i) Mma<DT>::run(acc, krow[2 * i], a[i]);
      // hidden keys (past the end of the split or past the row's causal limit) weigh nothing, and a row that
      // sees no key of the tile keeps its state
      if (!__all(n_vis >= 32)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = acc_row(r, kg) < n_vis ? acc[r] : NEG_BIG;
      }
      float mx = acc[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc[r]);
      mx = half_pair_max(mx);  // both halves of the wave use one reference per row
      mx = mx > NEG_BIG ? mx * p.scale2 : NEG_BIG;  // the reference lives in the scaled (log2) domain; scale2 > 0
      if (__any(mx > m_ref)) {
        const float m_new = fmaxf(m_ref, mx);
        const float alpha = fast_exp2(m_ref - m_new);
        l_sum *= alpha;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
        m_ref = m_new;
      }
      // a row without a visible key so far subtracts nothing: its hidden logits give 2^(NEG_BIG * scale2) = 0
      const float m_sub = m_ref > NEG_BIG ? m_ref : 0.0f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        acc[r] = fast_exp2(fmaf(acc[r], p.scale2, -m_sub));
        l_sum += acc[r];
      }
#pragma unroll
      for (int s = 0; s < RUNS; ++s) {
        uint4 pb;
        if (DT == DT_BF16) {
          pb = make_uint4(pack_bf16(acc[8 * s], acc[8 * s + 1]), pack_bf16(acc[8 * s + 2], acc[8 * s + 3]),
                          pack_bf16(acc[8 * s + 4], acc[8 * s + 5]), pack_bf16(acc[8 * s + 6], acc[8 * s + 7]));
        } else {
          pb = make_uint4(__float_as_uint(acc[4 * s]), __float_as_uint(acc[4 * s + 1]),
                          __float_as_uint(acc[4 * s + 2]), __float_as_uint(acc[4 * s + 3]));
        }
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
          const uint4* vrow = sVT + (size_t)(dt * 32 + rl) * VTP;
          uint4 va;
          if (DT == DT_BF16) {
            va = vrow[nt * 4 + 2 * s + kg];  // registers 8s .. 8s+7 are keys 16s + 4kg + (0..3) and the same + 8: see store_vt
          } else {
            va = vrow[nt * 8 + 2 * s + kg];  // registers 4s .. 4s+3 are keys 8s + 4kg + (0..3)
          }
          Mma<DT>::run(o[dt], va, pb);
        }
      }
    }
    seg = nseg;
    kc0 = nkc;
    have = nhave;
  }

  l_sum = half_pair_sum(l_sum);
  // several waves share a row tile over different key tiles: their states meet in LDS (rows padded by four
  // floats against bank conflicts) and leave as one partial per split
  constexpr int OP = D + 4;
  float* sO = reinterpret_cast<float*>(smem);                       // [8 waves][32 rows][OP]
  float2* sML = reinterpret_cast<float2*>(sO + ATT_WAVES * 32 * OP);  // [8 waves][32 rows]
  lds_barrier();  // the chunk buffers are free
  {
    float* dst = sO + (size_t)(wave * 32 + rl) * OP;
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
        *reinterpret_cast<float4*>(dst + dt * 32 + 8 * q4 + 4 * kg) =
            make_float4(o[dt][4 * q4], o[dt][4 * q4 + 1], o[dt][4 * q4 + 2], o[dt][4 * q4 + 3]);
    if (kg == 0) sML[wave * 32 + rl] = make_float2(m_ref, l_sum);
  }
  lds_barrier();
  const int n_rtw = ATT_WAVES >> p.wprt_log;  // row tiles of this workgroup
  for (int e = tid; e < n_rtw * 32 * (D / 4); e += ATT_THREADS) {
    const int d4 = e % (D / 4), rr = e / (D / 4);  // rr = row tile * 32 + row in tile
    const int row2 = qg * ATT_ROWS + rr;
    if (row2 >= p.m_rows) continue;
    const int w0 = (rr >> 5) << p.wprt_log, r2 = rr & 31;  // first wave of the tile
    float mx = NEG_BIG;
    for (int k = 0; k < wprt; ++k) mx = fmaxf(mx, sML[(w0 + k) * 32 + r2].x);
    float l = 0.0f;
    float4 acc = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int k = 0; k < wprt; ++k) {
      const float2 ml = sML[(w0 + k) * 32 + r2];
      const float wgt = fast_exp2(ml.x - mx);
      const float4 ov = *reinterpret_cast<const float4*>(sO + (size_t)((w0 + k) * 32 + r2) * OP + d4 * 4);
      l = fmaf(ml.y, wgt, l);
      acc.x = fmaf(ov.x, wgt, acc.x);
      acc.y = fmaf(ov.y, wgt, acc.y);
      acc.z = fmaf(ov.z, wgt, acc.z);
      acc.w = fmaf(ov.w, wgt, acc.w);
    }
    const size_t at = ((size_t)h * p.n_parts + split) * p.m_rows + row2;
    if (d4 == 0) p.part_ml[at] = make_float2(mx, l);
    *reinterpret_cast<float4*>(p.part_o + at * D + d4 * 4) = acc;
  }
}

// The same pass for launches in which every wave owns a row tile (8 or more query rows tiles per KV head: window
// rows, whole blocks), arranged so that the matrix unit and the vector unit work at the same time.  The keys of
// a chunk are complete tiles (hidden keys are masked, a tile nobody sees costs its arithmetic), so the tile loop
// has no early exits and is unrolled: the logits of tile t+1 are issued before the softmax of tile t, whose
// exponentials then run while the matrix unit multiplies.  Chunks alternate between two LDS stages: the next
// chunk, prefetched into registers while the current one is worked on, is stored after the chunk's last tile,
// so one barrier per chunk suffices (every wave has left the stage that is overwritten a barrier ago).
template <int DT>
__host__ __device__ constexpr int rows_chunk_keys() { return DT == DT_BF16 ? 128 : 64; }

template <int DT, int D>
__global__ __launch_bounds__(ATT_THREADS) void attend_rows_kernel(AttendParams p) {
  constexpr int ES = DT == DT_BF16 ? 2 : 4;
  constexpr int CH = D * ES / 16;             // 16-byte chunks per row
  constexpr int NCH = CH / 2;
  constexpr int CHP = CH + 1;                 // K row pitch in chunks (odd)
  constexpr int KC = rows_chunk_keys<DT>();   // keys per LDS chunk
  constexpr int EPC = 16 / ES;                // elements per 16-byte chunk
  constexpr int VTP = KC / EPC + 1;           // V^T row pitch in chunks (odd)
  constexpr int KL = KC * CH / ATT_THREADS;   // 16-byte loads per thread, tensor and chunk
  constexpr int NDT = D / 32;                 // 32-wide tiles of the head dimension
  constexpr int TPC = KC / 32;                // key tiles per chunk
  constexpr int RUNS = 32 / (2 * EPC);        // operand chunks per lane and 32-key tile in P.V
  constexpr int K_ROWS_PER_LOAD = ATT_THREADS / CH;
  constexpr int V_GROUPS_PER_LOAD = ATT_THREADS / (EPC * CH);
  // bf16: V stays key-major in LDS (rows of CH chunks + 2: a 4-key x 32-byte transposing read touches every bank
  // once) and ds_read_b64_tr_b16 delivers it transposed; fp32 has no such read: V^T is built in registers
  constexpr bool TR = DT == DT_BF16;
  constexpr int VP = CH + 2;                  // V row pitch in chunks (bf16)
  constexpr int STAGE = KC * CHP + (TR ? KC * VP : D * VTP);   // uint4 per LDS stage: K [KC][CHP], then V [KC][VP] or V^T [D][VTP]
  static_assert(KL >= 1 && KL * ATT_THREADS == KC * CH, "chunk not a whole number of loads per thread");

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, rl = lane & 31, kg = lane >> 5;
  // consecutive indices stay on one XCD: the row groups and splits of a head share that XCD's L2
  const int idx = xcd_major(blockIdx.x, gridDim.x);
  const int split = idx % p.n_splits, qg = (idx / p.n_splits) % p.n_qgroups, h = idx / (p.n_splits * p.n_qgroups);
  const int row = qg * ATT_ROWS + wave * 32 + rl;

  extern __shared__ uint4 smem[];

  // the wave's 32 query rows, as the B operand of S^T
  uint4 a[NCH];
  int blk_end_lane;  // block keys [0, blk_end_lane) are visible to this lane's row
  {
    const int m = min(row, p.m_rows - 1);
    const int g = m / p.n_q, j = m - g * p.n_q;
    const char* ptr = p.q.base + (int64_t)(h * p.group + g) * p.q.stride_head + (int64_t)j * p.q.stride_row;
#pragma unroll
    for (int i = 0; i < NCH; ++i) a[i] = ld16(ptr + (2 * i + kg) * 16);
    blk_end_lane = max(0, min(p.s_t, p.diag + j + 1));
  }
  const int lo0 = min(split * p.keys_per_split, p.cache_len), hi0 = min(lo0 + p.keys_per_split, p.cache_len);
  int lo1 = 0, hi1 = 0;
  if (p.s_t > 0) {
    const int m0 = qg * ATT_ROWS, m1 = min(m0 + ATT_ROWS, p.m_rows) - 1;
    const int g0 = m0 / p.n_q, g1 = m1 / p.n_q;
    const int j_max = g0 == g1 ? m1 - g1 * p.n_q : p.n_q - 1;
    const int wg_end = max(0, min(p.s_t, p.diag + j_max + 1));
    lo1 = min(split * p.blk_keys_per_split, wg_end);
    hi1 = min(lo1 + p.blk_keys_per_split, wg_end);
  }

  const __amdgpu_buffer_rsrc_t ksrd0 = make_srd(p.k_cache + (int64_t)h * p.cache_stride_head, (uint32_t)p.cache_len * (uint32_t)p.row_bytes);
  const __amdgpu_buffer_rsrc_t vsrd0 = make_srd(p.v_cache + (int64_t)h * p.cache_stride_head, (uint32_t)p.cache_len * (uint32_t)p.row_bytes);
  const uint32_t kb_bytes = p.s_t > 0 ? (uint32_t)(p.s_t - 1) * (uint32_t)p.kb_stride_row + (uint32_t)p.row_bytes : 0u;
  const uint32_t vb_bytes = p.s_t > 0 ? (uint32_t)(p.s_t - 1) * (uint32_t)p.vb_stride_row + (uint32_t)p.row_bytes : 0u;
  const __amdgpu_buffer_rsrc_t ksrd1 = make_srd(p.k_blk + (int64_t)h * p.kb_stride_head, kb_bytes);
  const __amdgpu_buffer_rsrc_t vsrd1 = make_srd(p.v_blk + (int64_t)h * p.vb_stride_head, vb_bytes);
  const uint32_t k_row = tid / CH, k_col = tid % CH;
  const uint32_t v_i = tid % EPC, v_c = (tid / EPC) % CH, v_grp = tid / (EPC * CH);
  uint4 kpre[KL], vpre[KL];
  auto prefetch = [&](int seg, int kc0) {
    const __amdgpu_buffer_rsrc_t ksrd = seg ? ksrd1 : ksrd0, vsrd = seg ? vsrd1 : vsrd0;
    const uint32_t kstride = seg ? (uint32_t)p.kb_stride_row : (uint32_t)p.row_bytes;
    const uint32_t vstride = seg ? (uint32_t)p.vb_stride_row : (uint32_t)p.row_bytes;
#pragma unroll
    for (int u = 0; u < KL; ++u) {
      kpre[u] = buf_ld16(ksrd, (uint32_t)(kc0 + k_row + u * K_ROWS_PER_LOAD) * kstride + k_col * 16);
      if (TR) {
        vpre[u] = buf_ld16(vsrd, (uint32_t)(kc0 + k_row + u * K_ROWS_PER_LOAD) * vstride + k_col * 16);
      } else {
        const uint32_t key = (u * V_GROUPS_PER_LOAD + v_grp) * EPC + v_i;
        vpre[u] = buf_ld16(vsrd, (uint32_t)(kc0 + key) * vstride + v_c * 16);
      }
    }
  };
  auto store = [&](uint4* stage) {
    uint4* sK = stage;
    uint4* sV = stage + KC * CHP;
#pragma unroll
    for (int u = 0; u < KL; ++u) {
      sK[(k_row + u * K_ROWS_PER_LOAD) * CHP + k_col] = kpre[u];
      if (TR) {
        sV[(k_row + u * K_ROWS_PER_LOAD) * VP + k_col] = vpre[u];
      } else {
        store_vt<DT>(sV + (v_c * EPC + v_i) * VTP, u * V_GROUPS_PER_LOAD + v_grp, transpose_4x4_b32(vpre[u], lane));
      }
    }
  };
  // Transposing read of V (bf16).  Within 16 lanes, lane i hands in the address of 4 consecutive 16-bit values and
  // lane 4c + e receives value e of lanes c, c + 4, c + 8, c + 12.  Lane i points at key (i >> 2) of a run of four
  // keys and head-dimension offset 4 (i & 3), so lane l of the sixteen receives the four keys at head-dimension
  // offset l: the A operand of O^T += V^T P^T.  Byte offset of this lane's piece within a V stage, for key 0 of the
  // tile's first 16-key block and head-dimension tile 0:
  const uint32_t tr_off = (uint32_t)((4 * kg + ((lane & 15) >> 2)) * VP * 16 + ((lane >> 4) & 1) * 32 + (lane & 3) * 8);
  // the chunk after (seg, kc0): the next of the segment, else the first of the block's keys
  auto advance = [&](int& seg, int& kc0) -> bool {
    kc0 += KC;
    if (kc0 < (seg ? hi1 : hi0)) return true;
    if (seg == 0 && lo1 < hi1) {
      seg = 1;
      kc0 = lo1;
      return true;
    }
    return false;
  };
  auto logits = [&](const uint4* stage, int nt, f32x16& acc) {
    const uint4* krow = stage + (size_t)(nt * 32 + rl) * CHP + kg;
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) Mma<DT>::run(acc, krow[2 * i], a[i]);
  };

  // Two attempts at most.  In the first, a row's reference is its maximum over the first tile of the cache rows
  // and complete tiles of cache rows after it skip the maximum, the comparison and the rescaling (an fma, an
  // exponential and an add per logit are all that is left); sums that grow past 2^100 (a later logit far above
  // the first tile's) make the workgroup repeat the pass with a reference that follows the running maximum
  // everywhere, as the block's own keys (masked, and possibly a row's first visible keys) always do.
  float m_ref, l_sum;
  f32x16 o[NDT];
  int* redo = reinterpret_cast<int*>(smem + (size_t)2 * STAGE);  // one word behind the two stages
  if (tid == 0) *redo = 0;  // ordered before the writes after the first attempt by the barriers in between
#pragma unroll 1
  for (int attempt = 0; attempt < 2; ++attempt) {
  const bool fixed_ref = attempt == 0 && DT == DT_BF16;  // fp32 rows (512 bytes) leave no registers for a second tile body
  m_ref = NEG_BIG;
  l_sum = 0.0f;
#pragma unroll
  for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[dt][r] = 0.0f;

  int seg = lo0 < hi0 ? 0 : 1;
  int kc0 = seg ? lo1 : lo0;
  bool have = seg ? lo1 < hi1 : true;
  int nseg = seg, nkc = kc0;
  bool nhave = false;
  int cur = 0;
  if (have) {
    prefetch(seg, kc0);
    store(smem);
    nhave = advance(nseg, nkc);
    if (nhave) prefetch(nseg, nkc);  // in flight while the first chunk is worked on
    lds_barrier();
  }
  while (have) {
    const uint4* stage = smem + (size_t)cur * STAGE;
    const uint4* sVT = stage + KC * CHP;
    const char* sVb = reinterpret_cast<const char*>(sVT) + tr_off;
    const int lane_end = seg ? min(hi1, blk_end_lane) : hi0;  // end of the keys of this segment the lane's row sees
    f32x16 acc, acc_next;
    logits(stage, 0, acc);
#pragma unroll
    for (int nt = 0; nt < TPC; ++nt) {
      if (nt + 1 < TPC) logits(stage, nt + 1, acc_next);  // the matrix unit works on these during the exponentials below
      const int n_vis = lane_end - (kc0 + nt * 32);  // keys of this tile the lane's row sees (>= 32: all)
      // workgroup-uniform: a complete tile of cache rows that is not the pass's first
      if (fixed_ref && seg == 0 && kc0 + nt * 32 > lo0 && kc0 + nt * 32 + 32 <= hi0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          acc[r] = fast_exp2(fmaf(acc[r], p.scale2, -m_ref));
          l_sum += acc[r];
        }
      } else {
      if (!__all(n_vis >= 32)) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = acc_row(r, kg) < n_vis ? acc[r] : NEG_BIG;
      }
      float mx = acc[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc[r]);
      mx = half_pair_max(mx);  // both halves of the wave use one reference per row
      mx = mx > NEG_BIG ? mx * p.scale2 : NEG_BIG;  // the reference lives in the scaled (log2) domain; scale2 > 0
      if (__any(mx > m_ref)) {
        const float m_new = fmaxf(m_ref, mx);
        const float alpha = fast_exp2(m_ref - m_new);
        l_sum *= alpha;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
        m_ref = m_new;
      }
      // a row without a visible key so far subtracts nothing: its hidden logits give 2^(NEG_BIG * scale2) = 0
      const float m_sub = m_ref > NEG_BIG ? m_ref : 0.0f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        acc[r] = fast_exp2(fmaf(acc[r], p.scale2, -m_sub));
        l_sum += acc[r];
      }
      }
#pragma unroll
      for (int s = 0; s < RUNS; ++s) {
        uint4 pb;
        if (DT == DT_BF16) {
          pb = make_uint4(pack_bf16(acc[8 * s], acc[8 * s + 1]), pack_bf16(acc[8 * s + 2], acc[8 * s + 3]),
                          pack_bf16(acc[8 * s + 4], acc[8 * s + 5]), pack_bf16(acc[8 * s + 6], acc[8 * s + 7]));
        } else {
          pb = make_uint4(__float_as_uint(acc[4 * s]), __float_as_uint(acc[4 * s + 1]),
                          __float_as_uint(acc[4 * s + 2]), __float_as_uint(acc[4 * s + 3]));
        }
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
          const uint4* vrow = sVT + (size_t)(dt * 32 + rl) * VTP;
          uint4 va;
          if (TR) {
            // registers 8s .. 8s+3 are keys 16s + 4kg + (0..3), registers 8s+4 .. 8s+7 the same + 8
            const char* at = sVb + (size_t)((nt * 32 + 16 * s) * VP) * 16 + dt * 64;
            const uint2 lo = ds_read_tr16(at), hi = ds_read_tr16(at + 8 * VP * 16);
            va = make_uint4(lo.x, lo.y, hi.x, hi.y);
          } else if (DT == DT_BF16) {
            va = vrow[nt * 4 + 2 * s + kg];  // registers 8s .. 8s+7 are keys 16s + 4kg + (0..3) and the same + 8: see store_vt
          } else {
            va = vrow[nt * 8 + 2 * s + kg];  // registers 4s .. 4s+3 are keys 8s + 4kg + (0..3)
          }
          Mma<DT>::run(o[dt], va, pb);
        }
      }
      if (nt + 1 < TPC) acc = acc_next;
    }
    // the next chunk goes into the other stage, which every wave left before the previous barrier
    have = nhave;
    if (have) {
      store(smem + (size_t)(cur ^ 1) * STAGE);
      seg = nseg;
      kc0 = nkc;
      nhave = advance(nseg, nkc);
      if (nhave) prefetch(nseg, nkc);
      cur ^= 1;
      lds_barrier();
    }
  }
  if (!fixed_ref) break;
  // inf, NaN or large enough for O = sum p v to overflow next: repeat (decided for the workgroup: the pass has barriers)
  if (!(l_sum < 1.0e30f)) *redo = 1;
  __syncthreads();
  if (!*redo) break;
  }

  l_sum = half_pair_sum(l_sum);
  if (row >= p.m_rows) return;
  if (p.direct) {
    // one split: the state is final.  out = O / l, lse = (m + log2 l) ln 2; a row that saw no key gives zero and -inf
    const size_t at = (size_t)h * p.m_rows + row;
    const float inv = l_sum > 0.0f ? 1.0f / l_sum : 0.0f;
    if (kg == 0) p.out_lse[at] = l_sum > 0.0f ? (m_ref + fast_log2(l_sum)) * 0.6931471805599453f : -__builtin_inff();
    float* dst = p.out + at * D;
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4)
        st16_stream(dst + dt * 32 + 8 * q4 + 4 * kg,
                    make_uint4(__float_as_uint(o[dt][4 * q4] * inv), __float_as_uint(o[dt][4 * q4 + 1] * inv),
                               __float_as_uint(o[dt][4 * q4 + 2] * inv), __float_as_uint(o[dt][4 * q4 + 3] * inv)));
    return;
  }
  // the split's partial (reference, sum, unnormalised output)
  const size_t at = ((size_t)h * p.n_parts + split) * p.m_rows + row;
  if (kg == 0) p.part_ml[at] = make_float2(m_ref, l_sum);
  float* dst = p.part_o + at * D;
#pragma unroll
  for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4)
      *reinterpret_cast<float4*>(dst + dt * 32 + 8 * q4 + 4 * kg) =
          make_float4(o[dt][4 * q4], o[dt][4 * q4 + 1], o[dt][4 * q4 + 2], o[dt][4 * q4 + 3]);
}

// out = sum_p O_p 2^(m_p - M) / sum_p l_p 2^(m_p - M), lse = (M + log2 of that sum) ln 2.  One workgroup per row:
// D / 4 lanes across the head dimension times COMB_SLICES slices of the partials, each slice merged on the fly
// and the slices then through LDS.  Without any partial (empty cache) the output is zero, the normaliser -inf.
constexpr int COMB_SLICES = 8;
template <int D>
__global__ __launch_bounds__((D / 4) * COMB_SLICES) void attend_combine_kernel(AttendParams p) {
  constexpr int LPR = D / 4;  // lanes per row
  __shared__ float4 sAcc[COMB_SLICES][LPR];
  __shared__ float2 sMl[COMB_SLICES];
  const int row_lin = blockIdx.x;
  const int d4 = threadIdx.x % LPR, sl = threadIdx.x / LPR;
  const int h = row_lin / p.m_rows, m = row_lin - h * p.m_rows;
  const float2* ml = p.part_ml + (size_t)h * p.n_parts * p.m_rows + m;
  const float* po = p.part_o + ((size_t)h * p.n_parts * p.m_rows + m) * D + d4 * 4;
  float mx = NEG_BIG, l = 0.0f;
  float4 acc = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll 4
  for (int q = sl; q < p.n_parts; q += COMB_SLICES) {
    const float2 v = ml[(size_t)q * p.m_rows];
    const float4 ov = *reinterpret_cast<const float4*>(po + (size_t)q * p.m_rows * D);
    const float mn = fmaxf(mx, v.x);
    const float wa = fast_exp2(mx - mn), wb = fast_exp2(v.x - mn);
    l = l * wa + v.y * wb;
    acc.x = acc.x * wa + ov.x * wb;
    acc.y = acc.y * wa + ov.y * wb;
    acc.z = acc.z * wa + ov.z * wb;
    acc.w = acc.w * wa + ov.w * wb;
    mx = mn;
  }
  sAcc[sl][d4] = acc;
  if (d4 == 0) sMl[sl] = make_float2(mx, l);
  __syncthreads();
  if (sl != 0) return;
  float mt = NEG_BIG;
#pragma unroll
  for (int k = 0; k < COMB_SLICES; ++k) mt = fmaxf(mt, sMl[k].x);
  float lt = 0.0f;
  float4 at = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
#pragma unroll
  for (int k = 0; k < COMB_SLICES; ++k) {
    const float wgt = fast_exp2(sMl[k].x - mt);
    const float4 ov = sAcc[k][d4];
    lt = fmaf(sMl[k].y, wgt, lt);
    at.x = fmaf(ov.x, wgt, at.x);
    at.y = fmaf(ov.y, wgt, at.y);
    at.z = fmaf(ov.z, wgt, at.z);
    at.w = fmaf(ov.w, wgt, at.w);
  }
  const float inv = lt > 0.0f ? 1.0f / lt : 0.0f;
  *reinterpret_cast<float4*>(p.out + (size_t)row_lin * D + d4 * 4) = make_float4(at.x * inv, at.y * inv, at.z * inv, at.w * inv);
  if (d4 == 0) p.out_lse[row_lin] = lt > 0.0f ? (mt + fast_log2(lt)) * 0.6931471805599453f : -__builtin_inff();
}

// ---------------------------------------------------------------------------------------------
// The normaliser alone (out == null): log sum_i exp(q.k_i / sqrt(d)) of every query over the cache, which is
// all laserkv_set_row_lse needs.  No values are read, no output accumulators are kept, so 16 waves of 32
// rows each share a workgroup (512 rows: a GQA group's whole window reads the keys once).  Workgroup = (key
// split, group of 512 rows, KV head).  Keys pass through two LDS buffers in chunks (the next chunk's loads are
// issued before the current one is worked on and stored after it: one barrier per chunk).  K Q^T with the
// keys as the A operand puts a query row in a lane: each lane keeps (reference, sum of 2^(x - reference))
// over its keys; the reference is the maximum over the split's first tile, and a pass whose sums overflow is
// repeated with a reference that follows the running maximum.
// ---------------------------------------------------------------------------------------------
constexpr int LSE_WAVES = 16;
constexpr int LSE_THREADS = LSE_WAVES * 64;
constexpr int LSE_ROWS = 32 * LSE_WAVES;

template <int DT>
__host__ __device__ constexpr int lse_chunk_keys() { return DT == DT_BF16 ? 256 : 128; }

template <int DT, int D>
__global__ __launch_bounds__(LSE_THREADS) void attend_lse_kernel(AttendParams p) {
  constexpr int ES = DT == DT_BF16 ? 2 : 4;
  constexpr int CH = D * ES / 16;
  constexpr int NCH = CH / 2;
  constexpr int CHP = CH + 1;
  constexpr int KC = lse_chunk_keys<DT>();
  constexpr int KL = KC * CH / LSE_THREADS;
  constexpr int TPC = KC / 32;
  constexpr int ROWS_PER_LOAD = LSE_THREADS / CH;
  static_assert(KL >= 1 && KL * LSE_THREADS == KC * CH, "chunk not a whole number of loads per thread");

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, rl = lane & 31, kg = lane >> 5;
  const int split = blockIdx.x, rg = blockIdx.y, h = blockIdx.z;
  const int k_lo = split * p.keys_per_split;
  const int k_hi = min(k_lo + p.keys_per_split, p.cache_len);
  const int row = rg * LSE_ROWS + wave * 32 + rl;

  extern __shared__ uint4 smem[];  // two key buffers [KC][CHP]

  uint4 a[NCH];
  {
    const int m = min(row, p.m_rows - 1);
    const int g = div_w(m, p.nq_magic), j = m - g * p.n_q;
    const char* ptr = p.q.base + (int64_t)(h * p.group + g) * p.q.stride_head + (int64_t)j * p.q.stride_row;
#pragma unroll
    for (int i = 0; i < NCH; ++i) a[i] = ld16(ptr + (2 * i + kg) * 16);
  }
  const __amdgpu_buffer_rsrc_t ksrd =
      make_srd(p.k_cache + (int64_t)h * p.cache_stride_head, (uint32_t)p.cache_len * (uint32_t)p.row_bytes);
  const uint32_t k_row = tid / CH, k_col = tid % CH;
  uint4 kpre[KL];
  auto prefetch = [&](int kc0) {
#pragma unroll
    for (int u = 0; u < KL; ++u)
      kpre[u] = buf_ld16(ksrd, (uint32_t)(kc0 + k_row + u * ROWS_PER_LOAD) * (uint32_t)p.row_bytes + k_col * 16);
  };
  auto store = [&](uint4* buf) {
#pragma unroll
    for (int u = 0; u < KL; ++u) buf[(k_row + u * ROWS_PER_LOAD) * CHP + k_col] = kpre[u];
  };

  // One pass over the split's keys.  fixed_ref: the reference is the lane's maximum over the split's first tile and
  // is not raised by later complete tiles (one fma, one exponential, one add per logit and nothing else); a later
  // logit 2^7 above it overflows the sum, which the caller detects.  Otherwise the reference follows the maximum.
  float ref, sum;
  auto pass = [&](bool fixed_ref) {
    ref = NEG_BIG;
    sum = 0.0f;
    prefetch(k_lo);
    store(smem);
    lds_barrier();
    int cur = 0;
    for (int kc0 = k_lo; kc0 < k_hi; kc0 += KC) {
      const bool more = kc0 + KC < k_hi;
      if (more) prefetch(kc0 + KC);
      const uint4* sK = smem + (size_t)cur * KC * CHP;
#pragma unroll 1
      for (int nt = 0; nt < TPC; ++nt) {
        const int kbase = kc0 + nt * 32;
        if (kbase >= k_hi) break;  // workgroup-uniform
        f32x16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.0f;
        const uint4* krow = sK + (size_t)(nt * 32 + rl) * CHP + kg;
#pragma unroll
        for (int i = 0; i < NCH; ++i) Mma<DT>::run(acc, krow[2 * i], a[i]);
        const int n_vis = k_hi - kbase;  // keys of this tile inside the split (>= 32: all)
        if (n_vis >= 32 && fixed_ref && kbase > k_lo) {
#pragma unroll
          for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(acc[r], p.scale2, -ref));
        } else if (n_vis >= 32) {
          float mx = acc[0];
#pragma unroll
          for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc[r]);
          const float nref = fmaxf(ref, mx * p.scale2);  // scale2 > 0
          sum *= fast_exp2(ref - nref);
          ref = nref;
#pragma unroll
          for (int r = 0; r < 16; ++r) sum += fast_exp2(fmaf(acc[r], p.scale2, -ref));
        } else if (acc_row(0, kg) < n_vis) {  // the split's last tile: a lane that sees none of its keys keeps its state
          float mx = acc[0];
#pragma unroll
          for (int r = 1; r < 16; ++r) mx = acc_row(r, kg) < n_vis ? fmaxf(mx, acc[r]) : mx;
          const float nref = fmaxf(ref, mx * p.scale2);
          sum *= fast_exp2(ref - nref);
          ref = nref;
#pragma unroll
          for (int r = 0; r < 16; ++r) sum += acc_row(r, kg) < n_vis ? fast_exp2(fmaf(acc[r], p.scale2, -ref)) : 0.0f;
        }
      }
      if (more) store(smem + (size_t)(cur ^ 1) * KC * CHP);
      cur ^= 1;
      lds_barrier();
    }
  };
  int* redo = reinterpret_cast<int*>(smem + (size_t)2 * KC * CHP);  // one word behind the two key buffers
  if (tid == 0) *redo = 0;  // ordered before the writes below by the barriers of the pass
  pass(true);
  // an overflowed sum (inf, or NaN once it was rescaled) anywhere in the workgroup: once more with a running maximum
  // (the decision is taken for the workgroup as a whole: the pass has barriers)
  if (!(sum < 3.0e38f)) *redo = 1;
  __syncthreads();
  if (*redo) pass(false);
  lse_merge(ref, sum, half_other(ref, kg), half_other(sum, kg));  // the two halves hold the same rows over different keys
  if (kg == 0 && row < p.m_rows) p.part_ml[((size_t)h * p.n_parts + split) * p.m_rows + row] = make_float2(ref, sum);
}

// lse = (M + log2 sum_p l_p 2^(m_p - M)) ln 2 per row; -inf without any partial (empty cache)
__global__ __launch_bounds__(256) void attend_lse_combine_kernel(AttendParams p) {
  const int row_lin = blockIdx.x * 256 + threadIdx.x;
  if (row_lin >= p.n_kv_heads * p.m_rows) return;
  const int h = row_lin / p.m_rows, m = row_lin - h * p.m_rows;
  const float2* ml = p.part_ml + (size_t)h * p.n_parts * p.m_rows + m;
  float mx = NEG_BIG;
#pragma unroll 8
  for (int q = 0; q < p.n_parts; ++q) mx = fmaxf(mx, ml[(size_t)q * p.m_rows].x);
  float l = 0.0f;
#pragma unroll 8
  for (int q = 0; q < p.n_parts; ++q) {
    const float2 v = ml[(size_t)q * p.m_rows];
    l = fmaf(v.y, fast_exp2(v.x - mx), l);
  }
  p.out_lse[row_lin] = l > 0.0f ? (mx + fast_log2(l)) * 0.6931471805599453f : -__builtin_inff();
}

// ---- host side ----
void attend_plan(int m_rows, int64_t cache_len, int s_t, int n_kv_heads, int n_cu, AttendPlan* plan) {
  const int n_qg = (m_rows + ATT_ROWS - 1) / ATT_ROWS;
  const int n_rt = (min(m_rows, ATT_ROWS) + 31) / 32;
  int rt_pow2 = 1, wprt_log = 3;
  while (rt_pow2 < n_rt) { rt_pow2 <<= 1; --wprt_log; }
  int n_splits = n_cu / (n_kv_heads * n_qg);
  n_splits = max(1, min(n_splits, ATT_MAX_SPLITS));
  // every split takes a share of the cache rows and a share of the block's keys
  int64_t kps = (cache_len + n_splits - 1) / n_splits;
  kps = max((int64_t)32, (kps + 31) / 32 * 32);
  int bps = (s_t + n_splits - 1) / n_splits;
  bps = max(32, (bps + 31) / 32 * 32);
  const int need_c = (int)((cache_len + kps - 1) / kps), need_b = (s_t + bps - 1) / bps;
  n_splits = max(need_c, need_b);  // 0: no key at all
  plan->n_qgroups = n_qg;
  plan->wprt_log = wprt_log;
  plan->n_splits = n_splits;
  plan->keys_per_split = (int)kps;
  plan->blk_keys_per_split = bps;
  plan->n_parts = n_splits;
  plan->direct = n_splits == 1 && wprt_log == 0;
}

void attend_lse_plan(int m_rows, int64_t cache_len, int n_kv_heads, int n_cu, AttendPlan* plan) {
  const int n_rg = (m_rows + LSE_ROWS - 1) / LSE_ROWS;
  int n_splits = n_cu / (n_kv_heads * n_rg);
  n_splits = max(1, min(n_splits, ATT_MAX_SPLITS));
  int64_t kps = (cache_len + n_splits - 1) / n_splits;
  kps = max((int64_t)32, (kps + 31) / 32 * 32);
  n_splits = cache_len > 0 ? (int)((cache_len + kps - 1) / kps) : 0;
  plan->n_qgroups = n_rg;
  plan->wprt_log = 0;
  plan->n_splits = n_splits;
  plan->keys_per_split = (int)kps;
  plan->blk_keys_per_split = 32;
  plan->n_parts = n_splits;
  plan->direct = 0;
}

size_t attend_workspace_bytes(const AttendPlan& plan, int m_rows, int n_kv_heads, int head_dim) {
  if (plan.direct) return 256;  // the kernel writes the result itself
  const size_t rows = (size_t)n_kv_heads * plan.n_parts * m_rows;
  return ((rows * head_dim * 4 + 255) & ~(size_t)255) + rows * 8 + 256;
}

template <int DT, int D, int KC>
static hipError_t launch_attend_kc(const AttendParams& p, hipStream_t st) {
  constexpr int ES = DT == DT_BF16 ? 2 : 4;
  constexpr size_t lds_chunk = ((size_t)KC * (D * ES / 16 + 1) + (size_t)D * (KC / (16 / ES) + 1)) * 16;
  constexpr size_t lds_merge = (size_t)ATT_WAVES * 32 * ((D + 4) * 4 + 8);  // the waves' states when they share row tiles
  constexpr size_t lds = lds_chunk > lds_merge ? lds_chunk : lds_merge;
  static_assert(lds <= 160 * 1024, "attention chunk does not fit the LDS");
  hipLaunchKernelGGL((attend_kernel<DT, D, KC>), dim3(p.n_splits * p.n_qgroups * p.n_kv_heads), dim3(ATT_THREADS), lds, st, p);
  return hipGetLastError();
}

template <int DT, int D>
static hipError_t launch_attend_t(const AttendParams& p, hipStream_t st) {
  if (p.n_splits > 0) {
    hipError_t e;
    if (p.wprt_log == 0) {
      constexpr int ES = DT == DT_BF16 ? 2 : 4;
      constexpr int KC = rows_chunk_keys<DT>();
      constexpr size_t v_stage = DT == DT_BF16 ? (size_t)KC * (D * ES / 16 + 2) : (size_t)D * (KC / (16 / ES) + 1);
      constexpr size_t lds = (size_t)2 * ((size_t)KC * (D * ES / 16 + 1) + v_stage) * 16 + 16;  // two stages and the redo flag
      static_assert(lds <= 160 * 1024, "two attention chunks do not fit the LDS");
      hipLaunchKernelGGL((attend_rows_kernel<DT, D>), dim3(p.n_splits * p.n_qgroups * p.n_kv_heads), dim3(ATT_THREADS), lds, st, p);
      e = hipGetLastError();
    } else {
      e = launch_attend_kc<DT, D, att_chunk_keys<DT>()>(p, st);
    }
    if (e != hipSuccess || p.direct) return e;
  }
  hipLaunchKernelGGL((attend_combine_kernel<D>), dim3(p.n_kv_heads * p.m_rows), dim3((D / 4) * COMB_SLICES), 0, st, p);
  return hipGetLastError();
}

template <int DT, int D>
static hipError_t launch_attend_lse_t(const AttendParams& p, hipStream_t st) {
  constexpr int ES = DT == DT_BF16 ? 2 : 4;
  constexpr size_t lds = (size_t)2 * lse_chunk_keys<DT>() * (D * ES / 16 + 1) * 16 + 16;  // two key buffers and the redo flag
  static_assert(lds <= 160 * 1024, "two key chunks do not fit the LDS");
  if (p.n_splits > 0) {
    hipLaunchKernelGGL((attend_lse_kernel<DT, D>), dim3(p.n_splits, p.n_qgroups, p.n_kv_heads), dim3(LSE_THREADS), lds, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const int n_rows = p.n_kv_heads * p.m_rows;
  hipLaunchKernelGGL(attend_lse_combine_kernel, dim3((n_rows + 255) / 256), dim3(256), 0, st, p);
  return hipGetLastError();
}

hipError_t launch_attend_lse(int dtype, int head_dim, const AttendParams& p, hipStream_t st) {
  if (dtype == DT_BF16 && head_dim == 128) return launch_attend_lse_t<DT_BF16, 128>(p, st);
  if (dtype == DT_BF16 && head_dim == 64) return launch_attend_lse_t<DT_BF16, 64>(p, st);
  if (dtype == DT_F32 && head_dim == 128) return launch_attend_lse_t<DT_F32, 128>(p, st);
  if (dtype == DT_F32 && head_dim == 64) return launch_attend_lse_t<DT_F32, 64>(p, st);
  return hipErrorInvalidValue;
}

hipError_t launch_attend(int dtype, int head_dim, const AttendParams& p, hipStream_t st) {
  if (dtype == DT_BF16 && head_dim == 128) return launch_attend_t<DT_BF16, 128>(p, st);
  if (dtype == DT_BF16 && head_dim == 64) return launch_attend_t<DT_BF16, 64>(p, st);
  if (dtype == DT_F32 && head_dim == 128) return launch_attend_t<DT_F32, 128>(p, st);
  if (dtype == DT_F32 && head_dim == 64) return launch_attend_t<DT_F32, 64>(p, st);
  return hipErrorInvalidValue;
}

template <int DT, int D>
static hipError_t attend_attr() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attend_kernel<DT, D, att_chunk_keys<DT>()>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attend_rows_kernel<DT, D>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attend_lse_kernel<DT, D>), hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  return e;
}

hipError_t init_attend_attributes() {
  hipError_t e = attend_attr<DT_BF16, 128>();
  if (e == hipSuccess) e = attend_attr<DT_BF16, 64>();
  if (e == hipSuccess) e = attend_attr<DT_F32, 128>();
  if (e == hipSuccess) e = attend_attr<DT_F32, 64>();
  return e;
}

}  // namespace lkv
