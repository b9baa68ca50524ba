// Decode attention kernels of the EasySpec draft hot path (gfx950): the vector-ALU split-KV kernel,
// the matrix-core kernel for groups of columns of one sequence, the merge of split-KV partials;
// how a launch cuts the contexts; and their launch wrappers.
#include "launch_common.hpp"

#include <limits.h>

namespace es {

// ------------------------------------------------------------------------------------------
// Decode attention over the KV caches of a set's layers, split along the context.
// One workgroup = (context chunk, KV head, layer x column); it serves the G query heads that
// share the KV head.  A K or V row (hd elements) is spread over LPS lanes, 16 bytes each, so a
// wave load covers SPW = 64/LPS consecutive slots (1 KB, coalesced).  Each wave walks its own
// contiguous run of slots in batches of IT loads per operand, all issued before the first is
// used, with a running (max, sum, accumulator) per query head: scores and probabilities never
// leave registers, since K and V fragments of a slot sit in the same lanes.  The four waves'
// states are combined through LDS; if the context has more than one chunk the workgroup
// writes a partial (max, sum, accumulator) per head and attn_merge_kernel combines the chunks.
// For bf16 caches with 128-element heads and four to eight query heads per KV head the scores come
// from the matrix cores instead (K rows staged through the wave's own LDS into MFMA A fragments,
// the queries as two bf16 terms): the vector ALUs keep the softmax of one head per lane and P.V.
// ------------------------------------------------------------------------------------------
struct AttnArgs {
  const float* Q;
  const void* kc;
  const void* vc;
  float* PO;
  float* PM;
  float* PL;
  void* AO;
  int layer0, Hq, Hkv, B, max_ctx;
  int CH;       // fixed-length cut (matrix-core kernel): slots per chunk
  int nch_ref;  // even cut (vector kernel, nb_ref > 0): chunks of a column of nb_ref batches
  int nb_ref;
  int direct;   // vector kernel: LDS holds the state of every slot group (see the kernel's last part)
  float scale;
};

// The split-KV cut of one column: its chunk count and the slot range [s0, s1) of chunk `chunk`
// (empty for chunk >= nch).  Fixed-length cut: chunks of CH slots.  Even cut: the column's
// units (of `unit` slots, the smallest step of a wave) are dealt to round(nb * nch_ref / nb_ref)
// chunks whose unit counts differ by at most one, so that a context of a power-of-two length
// plus a few drafted tokens does not leave a sliver of a chunk.
__host__ __device__ __forceinline__ void chunk_range(const AttnArgs& a, int n_slots, int unit, int chunk, int& nch, int& s0,
                                                     int& s1) {
  if (a.nb_ref == 0) {
    nch = (n_slots + a.CH - 1) / a.CH;
    s0 = chunk * a.CH;
    s1 = s0 + a.CH < n_slots ? s0 + a.CH : n_slots;
  } else {
    const int nb = (n_slots + unit - 1) / unit;
    nch = (nb * a.nch_ref + a.nb_ref / 2) / a.nb_ref;
    nch = nch > nb ? nb : nch;
    nch = nch < 1 ? 1 : nch;
    s0 = (int)((long)chunk * nb / nch) * unit;
    s1 = (int)((long)(chunk + 1) * nb / nch) * unit;
    s1 = s1 < n_slots ? s1 : n_slots;
  }
}

// The run [w0, w1) of wave `wave` of `nwv` inside the chunk [s0, s1): the chunk's units dealt evenly.
__host__ __device__ __forceinline__ void wave_range(int s0, int s1, int unit, int wave, int nwv, int& w0, int& w1) {
  const int n_units = (s1 - s0 + unit - 1) / unit;
  w0 = s0 + wave * n_units / nwv * unit;
  w1 = s0 + (wave + 1) * n_units / nwv * unit;
  w1 = w1 < s1 ? w1 : s1;
}

constexpr int kAttnIT = 8;       // loads in flight per operand per lane
constexpr int kAttnSmallIT = 2;  // the same for the short steps that finish a wave's share

// Sum over aligned groups of N lanes (8, 16 or 32), every lane of a group receiving the total,
// with data-parallel-primitive operand swizzles (lane^1 and lane^2 inside quads, then the
// mirrored lane of the other half of 8 and of 16 lanes) instead of LDS permutes.  Same operand
// pairs as an xor butterfly, hence the same bits.
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
template <int N>
__device__ __forceinline__ float group_sum(float v) {
  static_assert(N == 8 || N == 16 || N == 32, "group size");
  v += dpp_f32<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_f32<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_f32<0x141>(v);  // row_half_mirror
  if (N >= 16) v += dpp_f32<0x140>(v);  // row_mirror
  if (N >= 32) v += __shfl_xor(v, 16, 64);
  return v;
}

template <typename T, int HD>
struct AttnGeom {
  static constexpr int EPL = Tr<T>::EPL, LPS = HD / EPL, SPW = 64 / LPS;
  static constexpr int WAVE_SLOTS = kAttnIT * SPW;    // slots one wave covers per batch
  static constexpr int UNIT = kAttnSmallIT * SPW;     // and per small step: the granularity of the split
};

extern __shared__ float dyn_f[];

// TREE: the columns are nodes of token trees and carry a visibility mask; without it every
// slot up to the column's own is visible and the mask logic costs no registers.
template <typename T, int HD, int G, bool TREE>
__global__ __launch_bounds__(512) void attn_kernel(AttnArgs a, Cols c) {
  typedef AttnGeom<T, HD> Geo;
  constexpr int EPL = Geo::EPL, LPS = Geo::LPS, SPW = Geo::SPW, IT = kAttnIT;
  const int chunk = blockIdx.x, kvh = blockIdx.y;
  const int li = blockIdx.z / c.n, col = blockIdx.z % c.n;
  const int n_slots = c.pos[col] + 1;
  // slots below vis_base are all visible; slot vis_base + i (i < 64) only if bit i is set (the
  // column's row of a token tree's mask).  Causal columns have vis_base = n_slots.
  const int vbase = c.vis_base[col];
  const unsigned long long vmask = c.vis_mask[col];
  int nch, s0, s1;
  chunk_range(a, n_slots, Geo::UNIT, chunk, nch, s0, s1);
  if (chunk >= nch) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, NWV = blockDim.x >> 6;  // 4 or 8 waves
  const int sub = lane / LPS, e0 = (lane % LPS) * EPL;

  const size_t rowbase = (((size_t)(a.layer0 + li) * a.B + c.seq[col]) * a.Hkv + kvh) * (size_t)a.max_ctx;
  // wave-uniform row bases; a lane's fragment of slot s lies s * HD + e0 elements further (32-bit offsets)
  const char* kb = reinterpret_cast<const char*>(reinterpret_cast<const T*>(a.kc) + rowbase * HD);
  const char* vb = reinterpret_cast<const char*>(reinterpret_cast<const T*>(a.vc) + rowbase * HD);
  constexpr uint32_t ROW_BYTES = HD * sizeof(T);
  const uint32_t lane_byte = e0 * sizeof(T);
  const int HQ = a.Hq * HD;

  float q[G][EPL], acc[G][EPL], m_run[G], l_run[G];
  // one head per lane (see the batch code): running maximum and sum of that head only
  // ... and, for bf16 caches and four to eight query heads per KV head, the scores themselves from the
  // matrix cores: a tile of 16 slots x 32 elements of K is the A operand, the queries (two bf16 terms,
  // hi and lo, one product each) the B operand with the heads repeated over the 16 columns.  With four
  // heads lane l receives the score of head 2 (l & 1) + ((l >> 1) & 1), the head the vector path leaves
  // there, and probabilities travel as quad broadcasts; with more, lane l has head l % 8 and the
  // probabilities of a batch go through a few hundred bytes of the wave's LDS, where every lane of a
  // slot's row reads all heads' values back (same address for the whole row: a broadcast).
  constexpr bool kScoresByMfma = LPS == 16 && G >= 4 && std::is_same<T, bf16_t>::value;
  constexpr bool kHeadPerLane = (G == 4 && LPS == 16) || kScoresByMfma;
  constexpr bool kQuadHeads = G == 4;
  constexpr int QKT = kScoresByMfma ? HD / 32 : 1;
  // per slot row (sub): 8 heads x 8 probabilities, 8 rescale factors, 4 floats of padding (bank spread)
  constexpr int kShareRow = 76;
  bf16x8 qh[QKT], ql[QKT];
  float m1 = -INFINITY, l1 = 0.f;
  const bool odd1 = lane & 1, odd2 = lane & 2;
  const int head_l = kQuadHeads ? 2 * (lane & 1) + ((lane >> 1) & 1) : min(lane & 7, G - 1);  // this lane's head
  // the lane's B fragments of the queries: requested here, split into their two bf16 terms only after the
  // wave's first K and V rows have been requested too (split_q), so that the two latencies overlap
  float q_raw[QKT][8];
  if constexpr (kScoresByMfma) {
    const float* qp = a.Q + ((size_t)li * kMaxCols + col) * HQ + (kvh * G + head_l) * HD + (lane >> 4) * 8;
#pragma unroll
    for (int kt = 0; kt < QKT; ++kt)
#pragma unroll
      for (int e = 0; e < 8; ++e) q_raw[kt][e] = qp[kt * 32 + e];
  }
  auto split_q = [&] {
#pragma unroll
    for (int kt = 0; kt < QKT; ++kt) split_bf16x8(q_raw[kt], qh[kt], ql[kt]);
  };
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const float* qp = a.Q + ((size_t)li * kMaxCols + col) * HQ + (kvh * G + g) * HD + e0;
#pragma unroll
    for (int j = 0; j < EPL; ++j) {
      if constexpr (!kScoresByMfma) q[g][j] = qp[j];
      acc[g][j] = 0.f;
    }
    m_run[g] = -INFINITY;
    l_run[g] = 0.f;
  }

  // The chunk's units are dealt evenly to the waves, each taking a contiguous run [w0, w1): full
  // batches of IT loads per operand (all issued before the first is used) while more than two
  // small steps' worth is left, then small steps, so that a wave's arithmetic follows its share
  // of the slots.  Slots past w1 fetch the run's last row instead (their scores are discarded
  // below): unconditional loads, no branch per load.
  int w0, w1;
  wave_range(s0, s1, Geo::UNIT, wave, NWV, w0, w1);
  auto fetch_k = [&](auto n_loads, int base, u32x4* kr) {
#pragma unroll
    for (int j = 0; j < decltype(n_loads)::value; ++j) {
      const int s = min(base + j * SPW + sub, w1 - 1);
      kr[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kb + ((uint32_t)s * ROW_BYTES + lane_byte)));
    }
  };
  auto fetch_v = [&](auto n_loads, int base, u32x4* vr) {
#pragma unroll
    for (int j = 0; j < decltype(n_loads)::value; ++j) {
      const int s = min(base + j * SPW + sub, w1 - 1);
      vr[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vb + ((uint32_t)s * ROW_BYTES + lane_byte)));
    }
  };
  // One batch: kr, vr hold its K and V rows.  `staged` runs once the K registers are free again (matrix-core
  // scores only: the rows sit in LDS by then), which is where the next batch is requested.
  auto consume = [&](auto n_loads, int base, u32x4* kr, const u32x4* vr, auto&& staged) {
    constexpr int N = decltype(n_loads)::value;
    // K for the matrix cores: tile t holds 16 slots; A row r = lane % 16 carries slot
    // (r % 4) * 4 + r / 4 of the tile, so that the score of the slot this lane's V load j = 4 t + i
    // brings (slot 4 i + sub of the tile) comes out in this lane, element i of the tile's result.
    // The rows are loaded whole (coalesced, as for the vector products) and turned into A fragments
    // through the wave's own 8 KB of LDS, the 16-byte pieces of slot row s XORed by s % 16 so that
    // neither the row-wise stores nor the fragment reads meet a bank twice.
    constexpr int NT = kScoresByMfma ? (N + 3) / 4 : 1;
    u32x4 ka[NT][QKT];
    if constexpr (kScoresByMfma) {
      u32x4* stage = reinterpret_cast<u32x4*>(dyn_f) + wave * (IT * SPW * LPS);
#pragma unroll
      for (int j = 0; j < N; ++j) stage[stage_store_piece(lane, j)] = kr[j];
      __builtin_amdgcn_wave_barrier();  // LDS operations of one wave execute in order: no wait is needed
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int kt = 0; kt < QKT; ++kt) ka[t][kt] = stage[stage_fetch_piece(lane, t, kt)];
      __builtin_amdgcn_wave_barrier();  // the reads are issued before the next batch's stores
      staged();
    }
    if constexpr (kHeadPerLane) {
      // Four query heads over a 16-lane row: instead of four row-wide sums per slot, the lanes
      // trade partial dot products pairwise so that lane l ends up with the row's total for head
      // 2 (l & 1) + ((l >> 1) & 1) alone; the softmax arithmetic is then done once per lane
      // (one head) and the probability of head g comes back to the row's other lanes as a
      // quad broadcast on its way into the P.V products.
      float sc1[N];
      f32x4 st[NT];
      if constexpr (kScoresByMfma) {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          f32x4 s_hi = {0.f, 0.f, 0.f, 0.f}, s_lo = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int kt = 0; kt < QKT; ++kt) {
            s_hi = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[t][kt]), qh[kt], s_hi, 0, 0, 0);
            s_lo = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[t][kt]), ql[kt], s_lo, 0, 0, 0);
          }
          st[t] = s_hi + s_lo;
        }
      }
#pragma unroll
      for (int j = 0; j < N; ++j) {
        const int s = base + j * SPW + sub;
        const bool valid = (int)(s < w1) & (int)(!TREE || (int)(s < vbase) | (int)((vmask >> ((s - vbase) & 63)) & 1ull));  // straight-line
        if constexpr (kScoresByMfma) {
          sc1[j] = valid ? st[j / 4][j % 4] * a.scale : -INFINITY;
        } else {
          float kv[EPL];
          unpack<T>(kr[j], kv);
          float d[4];
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            d[g] = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) d[g] += q[g][e] * kv[e];
          }
          const float t0 = (odd1 ? d[2] : d[0]) + dpp_f32<0xB1>(odd1 ? d[0] : d[2]);  // lane ^ 1
          const float t1 = (odd1 ? d[3] : d[1]) + dpp_f32<0xB1>(odd1 ? d[1] : d[3]);
          float v = (odd2 ? t1 : t0) + dpp_f32<0x4E>(odd2 ? t0 : t1);                  // lane ^ 2
          v += dpp_f32<0x124>(v);  // row_ror:4
          v += dpp_f32<0x128>(v);  // row_ror:8
          sc1[j] = valid ? v * a.scale : -INFINITY;
        }
      }
      float bm = sc1[0];
#pragma unroll
      for (int j = 1; j < N; ++j) bm = fmaxf(bm, sc1[j]);
      const float m_new = fmaxf(m1, bm);
      const float m_ref = m_new == -INFINITY ? 0.f : m_new;  // see the general path below
      const float alpha = __expf(m1 - m_ref);
      m1 = m_new;
      l1 *= alpha;
      if constexpr (kQuadHeads) {
        const float al[4] = {dpp_f32<0x00>(alpha), dpp_f32<0xAA>(alpha), dpp_f32<0x55>(alpha), dpp_f32<0xFF>(alpha)};
#pragma unroll
        for (int g = 0; g < 4; ++g)
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[g][e] *= al[g];
#pragma unroll
        for (int j = 0; j < N; ++j) {
          float vv[EPL];
          unpack<T>(vr[j], vv);
          const float p = __expf(sc1[j] - m_ref);  // 0 for slots past the end or masked
          l1 += p;
          // head g sits in quad lane 0, 2, 1, 3 for g = 0 .. 3
          const float pg[4] = {dpp_f32<0x00>(p), dpp_f32<0xAA>(p), dpp_f32<0x55>(p), dpp_f32<0xFF>(p)};
#pragma unroll
          for (int g = 0; g < 4; ++g)
#pragma unroll
            for (int e = 0; e < EPL; ++e) acc[g][e] += pg[g] * vv[e];
        }
      } else {
        // lanes 0..7 of a slot row put their head's probabilities and rescale factor into the wave's LDS
        // (the K tiles are in registers by now); every lane then reads all heads' values of its row
        constexpr int NP = (N + 3) / 4;  // 16-byte pieces of probabilities per head
        float* share = dyn_f + wave * (IT * SPW * LPS * 4) + sub * kShareRow;
        float pj[4 * NP];
#pragma unroll
        for (int j = 0; j < 4 * NP; ++j) {
          pj[j] = j < N ? __expf(sc1[j < N ? j : 0] - m_ref) : 0.f;  // 0 for slots past the end or masked
          l1 += pj[j];
        }
        if ((lane & 8) == 0) {
#pragma unroll
          for (int q4 = 0; q4 < NP; ++q4)
            *reinterpret_cast<f32x4*>(share + (lane & 7) * 8 + 4 * q4) = f32x4{pj[4 * q4], pj[4 * q4 + 1], pj[4 * q4 + 2], pj[4 * q4 + 3]};
          share[64 + (lane & 7)] = alpha;
        }
        __builtin_amdgcn_wave_barrier();  // LDS operations of one wave execute in order
        const f32x4 al0 = *reinterpret_cast<const f32x4*>(share + 64), al1 = *reinterpret_cast<const f32x4*>(share + 68);
        const float al[8] = {al0[0], al0[1], al0[2], al0[3], al1[0], al1[1], al1[2], al1[3]};
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
          for (int e = 0; e < EPL; ++e) acc[g][e] *= al[g];
#pragma unroll
        for (int q4 = 0; q4 < NP; ++q4) {  // four slots' probabilities of every head at a time (registers)
          f32x4 pg[G];
#pragma unroll
          for (int g = 0; g < G; ++g) pg[g] = *reinterpret_cast<const f32x4*>(share + g * 8 + 4 * q4);
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const int j = 4 * q4 + jj;
            if (j < N) {
              float vv[EPL];
              unpack<T>(vr[j], vv);
#pragma unroll
              for (int g = 0; g < G; ++g)
#pragma unroll
                for (int e = 0; e < EPL; ++e) acc[g][e] += pg[g][jj] * vv[e];
            }
          }
        }
        __builtin_amdgcn_wave_barrier();  // the reads are issued before the next batch's K rows overwrite the place
      }
      return;
    }
    float sc[N][G], m_use[G];
#pragma unroll
    for (int j = 0; j < N; ++j) {
      const int s = base + j * SPW + sub;
      const bool valid = (int)(s < w1) & (int)(!TREE || (int)(s < vbase) | (int)((vmask >> ((s - vbase) & 63)) & 1ull));  // straight-line
      float kv[EPL];
      unpack<T>(kr[j], kv);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float dot = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) dot += q[g][e] * kv[e];
        dot = group_sum<LPS>(dot);
        sc[j][g] = valid ? dot * a.scale : -INFINITY;
      }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float bm = sc[0][g];
#pragma unroll
      for (int j = 1; j < N; ++j) bm = fmaxf(bm, sc[j][g]);
      // The running maximum belongs to the slot group (the LPS lanes that share slots), not to the
      // wave: no cross-lane traffic per batch; the groups are brought to a common reference once,
      // after the loop.  A group whose slots so far were all past the end or masked still has
      // -inf: the exponentials then take 0 as reference and give 0 instead of exp(-inf + inf).
      const float m_new = fmaxf(m_run[g], bm);
      const float m_ref = m_new == -INFINITY ? 0.f : m_new;
      const float alpha = __expf(m_run[g] - m_ref);  // exp(-inf) = 0 on the first batch
      m_run[g] = m_new;
      m_use[g] = m_ref;
      l_run[g] *= alpha;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] *= alpha;
    }
#pragma unroll
    for (int j = 0; j < N; ++j) {
      float vv[EPL];
      unpack<T>(vr[j], vv);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float p = __expf(sc[j][g] - m_use[g]);  // 0 for slots past the end or masked
        l_run[g] += p;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] += p * vv[e];
      }
    }
  };
  auto process = [&](auto n_loads, int base) {
    u32x4 kr[decltype(n_loads)::value], vr[decltype(n_loads)::value];
    fetch_k(n_loads, base, kr);
    fetch_v(n_loads, base, vr);
    consume(n_loads, base, kr, vr, [] {});
  };
  int base = w0;  // wave-uniform, like the loop conditions
  constexpr std::integral_constant<int, IT> kFull{};
  auto full_batch_at = [&](int b) { return w1 - b > 2 * Geo::UNIT; };
  if constexpr (kScoresByMfma) {
    if (full_batch_at(base)) {
      u32x4 kr[IT], vr[IT];
      fetch_k(kFull, base, kr);
      fetch_v(kFull, base, vr);
      split_q();
      if constexpr (kQuadHeads) {
        // With the scores on the matrix cores the vector arithmetic of a batch no longer hides the
        // latency of the next one's loads behind other waves' work, so a wave keeps two batches in
        // flight: K of the next batch goes into the registers the staging has just freed, V into a
        // second set of registers.  (More heads: no registers left for that set.)
        u32x4 vn[IT];
        while (full_batch_at(base + Geo::WAVE_SLOTS)) {  // another full batch follows: request it, work on this one
          const int next = base + Geo::WAVE_SLOTS;
          consume(kFull, base, kr, vr, [&] {
            fetch_k(kFull, next, kr);
            fetch_v(kFull, next, vn);
            asm volatile("" ::: "memory");  // the requests stay here: the compiler would sink them to their first use
          });
          base = next;
#pragma unroll
          for (int j = 0; j < IT; ++j) vr[j] = vn[j];
        }
      }
      consume(kFull, base, kr, vr, [] {});  // four heads: the wave's last full batch
      base += Geo::WAVE_SLOTS;
    } else {
      split_q();
    }
  }
  for (; full_batch_at(base); base += Geo::WAVE_SLOTS) process(kFull, base);
  for (; base < w1; base += Geo::UNIT) process(std::integral_constant<int, kAttnSmallIT>{}, base);

  if constexpr (kHeadPerLane && !kQuadHeads) {  // back to every lane holding all heads' maximum and sum: through LDS
    float* share = dyn_f + wave * (IT * SPW * LPS * 4) + sub * kShareRow;
    if ((lane & 8) == 0) {
      share[lane & 7] = m1;
      share[8 + (lane & 7)] = l1;
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int g = 0; g < G; ++g) {
      m_run[g] = share[g];
      l_run[g] = share[8 + g];
    }
  }
  if constexpr (kScoresByMfma) __syncthreads();  // the combination below reuses the LDS the K tiles went through
  if constexpr (kHeadPerLane && kQuadHeads) {  // back to every lane holding all four heads' maximum and sum
    const float mm[4] = {dpp_f32<0x00>(m1), dpp_f32<0xAA>(m1), dpp_f32<0x55>(m1), dpp_f32<0xFF>(m1)};
    const float ll[4] = {dpp_f32<0x00>(l1), dpp_f32<0xAA>(l1), dpp_f32<0x55>(l1), dpp_f32<0xFF>(l1)};
#pragma unroll
    for (int g = 0; g < G; ++g) {
      m_run[g] = mm[g & 3];
      l_run[g] = ll[g & 3];
    }
  }

  // Combine the NWV * SPW slot groups of the workgroup (l_run counts each slot once per group,
  // every lane of a group holds the same value).  A group, or a whole chunk of a tree column,
  // may have seen no visible slot: its maximum is -inf, its sums 0, and its weight below 0.
  const size_t arow = (size_t)li * kMaxCols + col;
  auto emit = [&](int g, int e, float m, float l, float o0, float o1) {  // outputs e, e + 1 of head g
    const int head = kvh * G + g;
    if (nch == 1) {
      T* dst = reinterpret_cast<T*>(a.AO) + (size_t)li * Tr<T>::PARTS * kMaxCols * HQ;
      store_act1<T>(dst + xoff<T>(c.n, HQ, col, head * HD + e), (size_t)kMaxCols * HQ, o0 / l);
      store_act1<T>(dst + xoff<T>(c.n, HQ, col, head * HD + e + 1), (size_t)kMaxCols * HQ, o1 / l);
    } else {
      const size_t row = arow * a.Hq + head;
      *reinterpret_cast<float2*>(a.PO + (row * kMaxChunks + chunk) * HD + e) = make_float2(o0, o1);
      if (e == 0) {
        a.PM[row * kMaxChunks + chunk] = m;
        a.PL[row * kMaxChunks + chunk] = l;
      }
    }
  };
  if (a.direct) {
    // every group's state goes to LDS as it stands; each thread then folds all groups for two
    // adjacent outputs (no cross-lane traffic at all)
    const int P = NWV * SPW, p = wave * SPW + sub;
    float* w_acc = dyn_f;              // [P][G][HD]
    float* w_m = dyn_f + P * G * HD;   // [G][P]
    float* w_l = w_m + G * P;          // [G][P]
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
      for (int e = 0; e < EPL; e += 4)
        *reinterpret_cast<f32x4*>(w_acc + (p * G + g) * HD + e0 + e) = f32x4{acc[g][e], acc[g][e + 1], acc[g][e + 2], acc[g][e + 3]};
    }
    if (lane % LPS == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        w_m[g * P + p] = m_run[g];
        w_l[g * P + p] = l_run[g];
      }
    }
    __syncthreads();
    for (int idx = tid; idx < G * HD / 2; idx += blockDim.x) {
      const int g = idx / (HD / 2), e = (idx % (HD / 2)) * 2;
      float m = w_m[g * P];
      for (int q = 1; q < P; ++q) m = fmaxf(m, w_m[g * P + q]);
      const float m_ref = m == -INFINITY ? 0.f : m;
      float l = 0.f, o0 = 0.f, o1 = 0.f;
      for (int q = 0; q < P; ++q) {  // in group order: the result does not depend on timing
        const float wgt = __expf(w_m[g * P + q] - m_ref);
        const float2 v = *reinterpret_cast<const float2*>(w_acc + (q * G + g) * HD + e);
        l += w_l[g * P + q] * wgt;
        o0 += v.x * wgt;
        o1 += v.y * wgt;
      }
      emit(g, e, m, l, o0, o1);
    }
  } else {
    // LDS too small for every group: the groups of a wave are combined with shuffles first
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mw = m_run[g];
#pragma unroll
      for (int off = LPS; off < 64; off <<= 1) mw = fmaxf(mw, __shfl_xor(mw, off, 64));
      const float rescale = m_run[g] == -INFINITY ? 0.f : __expf(m_run[g] - mw);
      m_run[g] = mw;
      l_run[g] *= rescale;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] *= rescale;
#pragma unroll
      for (int off = LPS; off < 64; off <<= 1) {
        l_run[g] += __shfl_xor(l_run[g], off, 64);
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] += __shfl_xor(acc[g][e], off, 64);
      }
    }
    float* w_acc = dyn_f;                 // [NWV][G][HD]
    float* w_m = dyn_f + NWV * G * HD;    // [NWV][G]
    float* w_l = w_m + NWV * G;           // [NWV][G]
    if (sub == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int e = 0; e < EPL; ++e) w_acc[(wave * G + g) * HD + e0 + e] = acc[g][e];
    }
    if (lane == 0) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        w_m[wave * G + g] = m_run[g];
        w_l[wave * G + g] = l_run[g];
      }
    }
    __syncthreads();
    for (int idx = tid; idx < G * HD / 2; idx += blockDim.x) {
      const int g = idx / (HD / 2), e = (idx % (HD / 2)) * 2;
      float m = w_m[g];
      for (int w = 1; w < NWV; ++w) m = fmaxf(m, w_m[w * G + g]);
      const float m_ref = m == -INFINITY ? 0.f : m;
      float l = 0.f, o0 = 0.f, o1 = 0.f;
      for (int w = 0; w < NWV; ++w) {
        const float wgt = __expf(w_m[w * G + g] - m_ref);
        l += w_l[w * G + g] * wgt;
        o0 += w_acc[(w * G + g) * HD + e] * wgt;
        o1 += w_acc[(w * G + g) * HD + e + 1] * wgt;
      }
      emit(g, e, m, l, o0, o1);
    }
  }
}

// ------------------------------------------------------------------------------------------
// Attention on the matrix cores (bf16 caches).  The query rows that share one KV head — the G
// heads of up to 16/G columns of one sequence (the tokens of a calibration, the nodes of a tree
// level; a single column in a plain draft step) — are the 16 columns of MFMA tiles, so K and V
// are read once per group of columns and the per-slot arithmetic leaves the vector ALUs:
//   S^T[slot][row]  = K[slot][:] . Q[row][:]      A = K (rows = slots), B = Q^T, two-term bf16 q
//   O^T[e][row]    += V^T[e][slot] P^T[slot][row]  A = V^T, B = P^T, two-term bf16 p
// Each wave walks its own sub-chunk of the context in super tiles of 64 slots and leaves one
// split-KV partial per query row (merged by attn_merge_kernel; written out directly if the
// column's whole context is one sub-chunk).  The slots of a super tile are dealt to the four
// S^T tiles so that lane (row r, quarter q) ends up with the 16 CONSECUTIVE slots q*16 .. q*16+15:
// the accumulator layout of S^T is then the B-operand layout of the P.V instruction, and a
// V^T fragment is 8 consecutive slots.  V is stored [slot][head_dim]; a wave transposes its
// 64 x head_dim tile through its own piece of LDS (XOR-swizzled pieces, read back with the
// transposing LDS read).  grid = (ceil(sub-chunks / waves), Hkv, k * groups), block = 64 * waves.
// ------------------------------------------------------------------------------------------
struct ColGroups {
  int32_t n;                // groups
  int32_t first[kMaxCols];  // first column of group i
  int32_t count[kMaxCols];  // its columns (consecutive, same sequence); count * G <= 16
};
constexpr int kMfmaAttnWaves = 4;
typedef short v4i16 __attribute__((ext_vector_type(4)));

template <int HD, bool TREE>
__global__ __launch_bounds__(64 * kMfmaAttnWaves) void attn_mfma_kernel(AttnArgs a, Cols c, ColGroups cg, int G) {
  constexpr int KT = HD / 32, ET = HD / 16, PIECES = HD / 8;
  extern __shared__ u32x4 dyn_v[];  // per wave: V tile [64 slots][PIECES] then K tile [16 slots][PIECES], 16-byte pieces, swizzled
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, NWV = blockDim.x >> 6;
  const int chunk = blockIdx.x * NWV + wave, kvh = blockIdx.y;
  const int li = blockIdx.z / cg.n, grp = blockIdx.z % cg.n;
  const int first = cg.first[grp], cnt = cg.count[grp];
  const int r = lane & 15, q4 = lane >> 4;  // query row (MFMA column) and quarter / k-group
  const bool row_ok = r < cnt * G;
  const int col = first + (row_ok ? r / G : 0), g = row_ok ? r % G : 0;
  int n_max = 0;         // slots the longest column of the group attends to
  int n_all = INT_MAX;   // slots below this one are visible to every column of the group
  for (int i = 0; i < cnt; ++i) {
    n_max = max(n_max, c.pos[first + i] + 1);
    n_all = min(n_all, TREE ? min(c.pos[first + i] + 1, c.vis_base[first + i]) : c.pos[first + i] + 1);
  }
  const int ws0 = chunk * a.CH;
  if (ws0 >= n_max) return;  // whole wave; nothing below synchronises across waves
  const int ws1 = min(ws0 + a.CH, n_max);
  const int n_slots = c.pos[col] + 1;  // of this lane's row
  const int vbase = c.vis_base[col];
  const unsigned long long vmask = c.vis_mask[col];
  const int HQ = a.Hq * HD;
  const size_t rowbase = (((size_t)(a.layer0 + li) * a.B + c.seq[first]) * a.Hkv + kvh) * (size_t)a.max_ctx;
  const bf16_t* kc = reinterpret_cast<const bf16_t*>(a.kc) + rowbase * HD;
  const u32x4* vc = reinterpret_cast<const u32x4*>(reinterpret_cast<const bf16_t*>(a.vc) + rowbase * HD);
  u32x4* vt = dyn_v + (size_t)wave * 80 * PIECES;
  u32x4* kt_lds = vt + 64 * PIECES;
  const u32x4* kc4 = reinterpret_cast<const u32x4*>(kc);

  // K and V rows of a super tile as they lie in memory (coalesced): fragment f = it*64 + lane of its
  // 64 x PIECES 16-byte pieces.  The registers are free again once their contents sit in LDS, so
  // the next super tile is requested while the current one is still being worked on; the first
  // one before the queries are fetched.
  // Loads are unconditional: a slot past the sub-chunk's end (only the last sub-chunk of the longest
  // column has any: sub-chunks are multiples of 64 slots) re-reads the last row; its scores are masked
  // below for every query row, so its probabilities are exact zeros.
  u32x4 kf[PIECES], vf[PIECES];
  auto request = [&](int base) {
#pragma unroll
    for (int it = 0; it < PIECES; ++it) {
      const int f = it * 64 + lane, sl = min(base + f / PIECES, ws1 - 1), piece = f % PIECES;
      kf[it] = __builtin_nontemporal_load(kc4 + (size_t)sl * PIECES + piece);
    }
#pragma unroll
    for (int it = 0; it < PIECES; ++it) {
      const int f = it * 64 + lane, sl = min(base + f / PIECES, ws1 - 1), piece = f % PIECES;
      vf[it] = __builtin_nontemporal_load(vc + (size_t)sl * PIECES + piece);
    }
  };
  request(ws0);

  // B operands of S^T: this row's query, hi and lo bf16 terms, k-group q4 of every k-tile
  bf16x8 qh[KT], ql[KT];
  {
    const float* qp = a.Q + ((size_t)li * kMaxCols + col) * HQ + (kvh * G + g) * HD + q4 * 8;
#pragma unroll
    for (int kt = 0; kt < KT; ++kt) {
      float x[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = row_ok ? qp[kt * 32 + e] : 0.f;
      split_bf16x8(x, qh[kt], ql[kt]);
    }
  }

  f32x4 o[ET];
#pragma unroll
  for (int et = 0; et < ET; ++et) o[et] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.f;  // l_run: this lane's 16 slots per super tile only

  for (int base = ws0; base < ws1; base += 64) {
    // V tile into LDS, the 32-byte blocks of slot s XORed by s % 4: the transposing reads below take
    // the same block of four consecutive slots at once, which then lie in different banks
#pragma unroll
    for (int it = 0; it < PIECES; ++it) {
      const int f = it * 64 + lane, sl = f / PIECES, piece = f % PIECES;
      vt[sl * PIECES + (piece ^ ((sl & 3) << 1))] = vf[it];
    }
    // scores of this lane's row against its 16 slots base + q4*16 + t*4 + i.  S^T tile t takes
    // the slots (m/4)*16 + t*4 + m%4, m = 0..15, as its A rows: their pieces go through LDS
    // (piece p of A row m stored at p ^ m, so that the 16 rows of one piece hit 16 different banks)
    float sc[4][4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
#pragma unroll
      for (int it = 0; it < PIECES; ++it) {
        const int f = it * 64 + lane, sl = f / PIECES, piece = f % PIECES;
        // slot sl belongs to tile (sl / 4) % 4; with 16 pieces per row that is it % 4 for every lane
        if (PIECES == 16 ? (it & 3) == t : ((sl >> 2) & 3) == t) {
          const int m = (sl >> 4) * 4 + (sl & 3);
          kt_lds[m * PIECES + (piece ^ (m & (PIECES - 1)))] = kf[it];
        }
      }
      __builtin_amdgcn_wave_barrier();  // LDS operations of one wave execute in order: no wait is needed
      f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kt = 0; kt < KT; ++kt) {
        const u32x4 ka = kt_lds[r * PIECES + ((kt * 4 + q4) ^ (r & (PIECES - 1)))];
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka), qh[kt], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka), ql[kt], acc, 0, 0, 0);
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float v = acc[i] * a.scale;
        if (base + 64 <= n_all) {  // wave-uniform: a super tile that every query row sees whole needs no mask
          sc[t][i] = v;            // (padding rows get finite scores of a zero query; they are never stored)
        } else {
          const int slot = base + q4 * 16 + t * 4 + i;
          // no short circuit: the shift amount is masked instead of guarded, so that this stays straight-line code
          const bool seen = !TREE || (int)(slot < vbase) | (int)((vmask >> ((slot - vbase) & 63)) & 1ull);
          const bool valid = (int)row_ok & (int)(slot < n_slots) & (int)seen;
          sc[t][i] = valid ? v : -INFINITY;
        }
      }
    }
    if (base + 64 < ws1) request(base + 64);  // both register sets are in LDS / consumed by now
    float bm = -INFINITY;
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) bm = fmaxf(bm, sc[t][i]);
    bm = fmaxf(bm, __shfl_xor(bm, 16, 64));  // the four quarters of a row must share the reference:
    bm = fmaxf(bm, __shfl_xor(bm, 32, 64));  // their slots are summed by one instruction below
    const float m_new = fmaxf(m_run, bm);
    const float m_ref = m_new == -INFINITY ? 0.f : m_new;  // nothing visible so far: exponentials give 0
    const float alpha = __expf(m_run - m_ref);
    m_run = m_new;
    l_run *= alpha;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {  // wave-uniform: once the running maxima have settled nothing is rescaled
#pragma unroll
      for (int et = 0; et < ET; ++et) o[et] *= alpha;
    }
    // B operands of P.V: MFMA number h takes slots q4*16 + h*8 .. +8 of this lane = tiles 2h, 2h+1
    bf16x8 ph[2], pl[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float pv[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        pv[j] = __expf(sc[2 * h + (j >> 2)][j & 3] - m_ref);
        l_run += pv[j];
      }
      split_bf16x8(pv, ph[h], pl[h]);
    }
    __builtin_amdgcn_wave_barrier();
    // A operands: V^T row e = et*16 + lane%16, the 8 slots q4*16 + h*8 + j, by the LDS transposing
    // read (ds_read_b64_tr_b16): in a group of 16 lanes, lane i offers the 8 bytes at its address
    // (4 elements of "row" i) and receives element i%4 of rows i/4, i/4 + 4, i/4 + 8, i/4 + 12.
    // With row 4j + c = (slot s0 + j, elements e0 + 4c .. +3), lane i receives V[s0 + j][e0 + i],
    // j = 0..3: four consecutive slots of its own V^T row.  Two reads per 8-slot k-group.
#pragma unroll
    for (int et = 0; et < ET; ++et) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        v4i16 half[2];
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
          const int slot = q4 * 16 + h * 8 + t2 * 4 + (r >> 2);  // this lane's row of the transposed block
          const int piece = (et * 2 + ((r & 3) >> 1)) ^ ((slot & 3) << 1);
          const char* src = reinterpret_cast<const char*>(vt) + slot * (HD * 2) + piece * 16 + (r & 1) * 8;
          half[t2] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16*)(src));
        }
        typedef short v8i16 __attribute__((ext_vector_type(8)));
        const v8i16 both = {half[0][0], half[0][1], half[0][2], half[0][3], half[1][0], half[1][1], half[1][2], half[1][3]};
        const bf16x8 va = __builtin_bit_cast(bf16x8, both);
        o[et] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, ph[h], o[et], 0, 0, 0);
        o[et] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pl[h], o[et], 0, 0, 0);
      }
    }
    __builtin_amdgcn_wave_barrier();  // the gathers are issued before the next tile's stores into the same piece of LDS
  }

  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  if (!row_ok || ws0 >= n_slots) return;  // padding rows; columns that end before this sub-chunk
  const int nch = (n_slots + a.CH - 1) / a.CH;
  const int head = kvh * G + g;
  if (nch == 1) {
#pragma unroll
    for (int et = 0; et < ET; ++et) {
      const int e = et * 16 + q4 * 4;
      bf16_t* dst = reinterpret_cast<bf16_t*>(a.AO) + (size_t)li * 2 * kMaxCols * HQ + xoff<bf16_t>(c.n, HQ, col, head * HD + e);
      store_act4<bf16_t>(dst, (size_t)kMaxCols * HQ, o[et][0] / l_run, o[et][1] / l_run, o[et][2] / l_run, o[et][3] / l_run);
    }
  } else {
    const size_t row = ((size_t)li * kMaxCols + col) * a.Hq + head;
#pragma unroll
    for (int et = 0; et < ET; ++et)
      *reinterpret_cast<f32x4*>(a.PO + (row * kMaxChunks + chunk) * HD + et * 16 + q4 * 4) = o[et];
    if (q4 == 0) {
      a.PM[row * kMaxChunks + chunk] = m_run;
      a.PL[row * kMaxChunks + chunk] = l_run;
    }
  }
}

// Merge the chunk partials of one (layer, column, query head), chunks in order.  Runs as its own
// launch: the kernel boundary is what makes the partials written by workgroups on other XCDs
// visible (a device-scope fence inside the attention kernel costs an L2 write-back per workgroup
// and was measured several times slower).  Columns whose context fits one chunk were finished by
// attn_kernel.  grid = (k * columns, Hq), block = HD: one thread per output element, one small
// workgroup per head, so that the launch is as wide as the partials allow and costs one memory
// latency whatever the number of heads that share a KV head.
template <typename T, int HD>
__global__ __launch_bounds__(HD) void attn_merge_kernel(AttnArgs a, Cols c) {
  __shared__ float s_w[kMaxChunks];   // exp(m_chunk - m); chunk count <= 64 = one lane each
  __shared__ float s_lw[kMaxChunks];  // the chunk's sum on the common reference
  const int li = blockIdx.x / c.n, col = blockIdx.x % c.n, head = blockIdx.y, e = threadIdx.x;
  const int n_slots = c.pos[col] + 1;
  int nch, s0_unused, s1_unused;
  chunk_range(a, n_slots, AttnGeom<T, HD>::UNIT, 0, nch, s0_unused, s1_unused);
  if (nch == 1) return;
  const int HQ = a.Hq * HD;
  const size_t row = ((size_t)li * kMaxCols + col) * a.Hq + head;
  // every load is issued up front: the first 16 chunk partials of this thread's output element (all
  // of them for contexts up to 16 chunks) together with the chunk maxima and sums
  const float* po = a.PO + row * kMaxChunks * HD + e;
  float pv[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) pv[u] = u < nch ? po[(size_t)u * HD] : 0.f;
  if (e < 64) {  // the first wave: one lane per chunk
    const float pm = e < nch ? a.PM[row * kMaxChunks + e] : -INFINITY;
    const float pl = e < nch ? a.PL[row * kMaxChunks + e] : 0.f;
    float m = pm;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
    const float wgt = __expf(pm - m);
    s_w[e] = wgt;
    s_lw[e] = pl * wgt;
  }
  __syncthreads();
  float tot = 0.f;  // in chunk order so that the result does not depend on a reduction tree
  for (int ch = 0; ch < nch; ++ch) tot += s_lw[ch];
  float o = 0.f;
#pragma unroll
  for (int u = 0; u < 16; ++u) o += pv[u] * (u < nch ? s_w[u] : 0.f);
  for (int c0 = 16; c0 < nch; c0 += 8) {
    float pw[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) pw[u] = c0 + u < nch ? po[(size_t)(c0 + u) * HD] : 0.f;  // independent loads
#pragma unroll
    for (int u = 0; u < 8; ++u) o += pw[u] * (c0 + u < nch ? s_w[c0 + u] : 0.f);
  }
  store_act1<T>(reinterpret_cast<T*>(a.AO) + (size_t)li * Tr<T>::PARTS * kMaxCols * HQ + xoff<T>(c.n, HQ, col, head * HD + e),
                (size_t)kMaxCols * HQ, o / tot);
}

template <typename T, int HD, bool TREE>
static void launch_attn_g(int G, dim3 grid, int nwv, hipStream_t st, AttnArgs a, const Cols& c) {
  // partial state of every slot group of the workgroup if that fits the default 64 KB of
  // dynamic LDS, else of every wave
  const int groups = nwv * AttnGeom<T, HD>::SPW;
  a.direct = (size_t)groups * G * (HD + 2) * sizeof(float) <= 65536 ? 1 : 0;
  const int sets = a.direct ? groups : nwv;
  size_t lds = (size_t)sets * G * (HD + 2) * sizeof(float);
  // scores from the matrix cores (four query heads per KV head, bf16 caches): 8 KB per wave for the K tiles
  if (G >= 4 && AttnGeom<T, HD>::LPS == 16 && std::is_same<T, bf16_t>::value)
    lds = std::max(lds, (size_t)nwv * kAttnIT * AttnGeom<T, HD>::SPW * HD * sizeof(T));
  const dim3 blk(64 * nwv);
  switch (G) {
    case 1: ES_LAUNCH((attn_kernel<T, HD, 1, TREE>), grid, blk, lds, st, a, c); break;
    case 2: ES_LAUNCH((attn_kernel<T, HD, 2, TREE>), grid, blk, lds, st, a, c); break;
    case 4: ES_LAUNCH((attn_kernel<T, HD, 4, TREE>), grid, blk, lds, st, a, c); break;
    case 7: ES_LAUNCH((attn_kernel<T, HD, 7, TREE>), grid, blk, lds, st, a, c); break;
    case 8: ES_LAUNCH((attn_kernel<T, HD, 8, TREE>), grid, blk, lds, st, a, c); break;
    default: break;  // rejected at create
  }
}

// Matrix-core attention or the vector-ALU kernel?  The MFMA kernel reads K and V once per group
// of columns of a sequence and does the per-slot arithmetic on the matrix cores, but its
// per-wave chain (LDS transposes between the two products) is longer; measured, it wins once a
// launch holds several columns of a sequence and enough (column, layer, slot) work: tree levels,
// long calibrations.  Single columns (plain draft steps) and short 1-layer launches stay on the
// vector kernel.  EASYSPEC_ATTN_MFMA = 0 / 2 forces never / always (bf16 only).
static bool attn_use_mfma(const Shape& s, const Cols& c, int n_set) {
  const int mode = env_int("EASYSPEC_ATTN_MFMA", 1);  // read at every call: tests switch it between contexts
  const long min_work = env_int("EASYSPEC_ATTN_MFMA_MIN", 30000);
  if (mode == 0 || s.dtype != 1) return false;
  if (mode == 2) return true;
  bool shared = false;
  int max_len = 1;
  for (int i = 0; i < c.n; ++i) {
    shared = shared || (i > 0 && c.seq[i] == c.seq[i - 1]);
    max_len = std::max(max_len, c.pos[i] + 1);
  }
  // a launch over one layer with fewer than 5 columns keeps too few waves busy on the matrix cores (the
  // partial buffers cap the sub-chunks at kMaxChunks): 4-token calibration at context 8192, 3778 us
  // against 3699 us with the vector kernel; with 5 tokens 3830 against 3872 us, with 6 3834 against 3999 us
  return shared && (long)n_set * c.n * max_len >= min_work && (n_set > 1 || c.n >= 5);
}

// Runs of consecutive columns of one sequence, cut so that a group's query rows (columns x G
// heads per KV head) fill at most the 16 columns of an MFMA tile.
static void group_columns(const Cols& c, int G, ColGroups& cg) {
  const int most = std::max(1, 16 / G);
  cg.n = 0;
  for (int i = 0; i < c.n;) {
    int j = i + 1;
    while (j < c.n && c.seq[j] == c.seq[i] && j - i < most) ++j;
    cg.first[cg.n] = i;
    cg.count[cg.n] = j - i;
    ++cg.n;
    i = j;
  }
}

AttnCut attn_cut(const Shape& s, const Cols& c, int n_set) {
  AttnCut cut;
  cut.mfma = attn_use_mfma(s, c, n_set);
  cut.chunk = 0;
  cut.nb_ref = 0;
  int max_len = 1;
  for (int i = 0; i < c.n; ++i) max_len = std::max(max_len, c.pos[i] + 1);
  // Short contexts: one piece of work per (layer, column, KV head) walks the whole context, which
  // saves the merge launch; two dependent launches cost more than the narrower launch loses.
  static const int single_max = env_int("EASYSPEC_ATTN_SINGLE", 256);
  if (cut.mfma) {
    // one wave per (group of columns, sub-chunk, KV head), kMfmaAttnWaves of them per workgroup,
    // walking its sub-chunk in super tiles of 64 slots: sub-chunks of a fixed length, grown until
    // their count fits the partial buffers and the launch is not cut finer than one workgroup per CU
    // (measured: 8-wide tree level 3061 -> 2997 us against two per CU)
    ColGroups cg;
    group_columns(c, s.Hq / s.Hkv, cg);
    const int unit = 64;
    if (max_len <= single_max) {
      cut.chunk = (max_len + unit - 1) / unit * unit;
      cut.n_chunks = 1;
      return cut;
    }
    static const long max_wg = env_int("EASYSPEC_ATTN_WG", 256);
    int ch = unit;
    auto nch = [&](int ch_) { return (max_len + ch_ - 1) / ch_; };
    while (ch < 1024 && (nch(ch) > kMaxChunks || (long)nch(ch) * s.Hkv * n_set * cg.n > max_wg * kMfmaAttnWaves)) ch *= 2;
    cut.chunk = ch;
    cut.n_chunks = nch(ch);
    return cut;
  }
  return attn_cut_vector(s, c, n_set);
}

AttnCut attn_cut_vector(const Shape& s, const Cols& c, int n_set) {
  AttnCut cut;
  cut.mfma = false;
  cut.chunk = 0;
  int max_len = 1;
  for (int i = 0; i < c.n; ++i) max_len = std::max(max_len, c.pos[i] + 1);
  static const int single_max = env_int("EASYSPEC_ATTN_SINGLE", 256);
  // Vector kernel: one workgroup of four waves per (chunk, KV head, layer, column).  Every column's
  // units (the slots of a wave's small step) are dealt evenly to its chunks (chunk_range) and a
  // chunk's units evenly to its waves, which work through them in full batches of four units and
  // up to two small steps.  The chunk count of the longest column is the one that minimises the
  // arithmetic of the busiest SIMD — (workgroups per CU, rounded up) x (cost of the busiest wave
  // of a workgroup) — and among equals the smallest (fewer partials to merge).
  const int lps = s.hd * (s.dtype == 1 ? 2 : 4) / 16;
  const int unit = kAttnSmallIT * (64 / lps);
  const int nb_max = (max_len + unit - 1) / unit;
  cut.nb_ref = nb_max;
  cut.n_chunks = 1;
  if (max_len <= single_max) return cut;
  const int forced = env_int("EASYSPEC_ATTN_NCH", 0);  // tests: a fixed count for the longest column, read at every call
  static const int n_cu = [] {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
    return n;
  }();
  // cost of a wave with u units, in tenths of a full batch: a small step does a quarter of a
  // batch's slots at about a third of its time
  constexpr int per_batch = kAttnIT / kAttnSmallIT;
  auto wave_cost = [](long u) {
    const long full = u / per_batch, rest = u % per_batch;
    return 10 * full + (rest == 0 ? 0 : rest <= 2 ? 3 * rest + 1 : 10);
  };
  long best = -1;
  for (int nch = forced > 0 ? std::min(forced, nb_max) : 2; nch <= std::min(kMaxChunks, nb_max); ++nch) {
    long wgs = 0;
    for (int i = 0; i < c.n; ++i) {
      const int nb = (c.pos[i] + 1 + unit - 1) / unit;
      wgs += std::max(1, std::min(nb, (nb * nch + nb_max / 2) / nb_max));
    }
    wgs *= (long)s.Hkv * n_set;
    const long per_cu = (wgs + n_cu - 1) / n_cu;
    const long per_wave = ((nb_max + nch - 1) / nch + 3) / 4;  // units of the busiest wave
    const long score = per_cu * wave_cost(per_wave);
    if (best < 0 || score < best) {
      best = score;
      cut.n_chunks = nch;
    }
    if (forced > 0) break;
  }
  return cut;
}

int attn_waves(const AttnCut& cut) { return cut.n_chunks == 1 ? 8 : 4; }

void attn_ranges(const Shape& s, const AttnCut& cut, int n_slots, int chunk, int wave, int* nch, int* w0, int* w1) {
  AttnArgs a;
  a.CH = cut.chunk; a.nch_ref = cut.n_chunks; a.nb_ref = cut.nb_ref;
  const int lps = s.hd * (s.dtype == 1 ? 2 : 4) / 16;
  const int unit = kAttnSmallIT * (64 / lps);
  int s0, s1;
  chunk_range(a, n_slots, unit, chunk, *nch, s0, s1);
  if (chunk >= *nch) {
    *w0 = *w1 = 0;
    return;
  }
  wave_range(s0, s1, unit, wave, attn_waves(cut), *w0, *w1);
}

void launch_attn(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, const AttnCut& cut, hipStream_t st) {
  const int n_chunks = cut.n_chunks;
  AttnArgs a;
  a.Q = b.Q; a.kc = b.kc; a.vc = b.vc; a.PO = b.PO; a.PM = b.PM; a.PL = b.PL; a.AO = b.AO;
  a.layer0 = layer0; a.Hq = s.Hq; a.Hkv = s.Hkv; a.B = s.B; a.max_ctx = s.max_ctx;
  a.CH = cut.chunk; a.nch_ref = cut.n_chunks; a.nb_ref = cut.nb_ref;
  a.scale = 1.0f / sqrtf((float)s.hd);
  const int G = s.Hq / s.Hkv;
  const dim3 grid(n_chunks, s.Hkv, n_set * c.n);
  // one chunk per context: eight waves share the whole context of a (layer, column, KV head) and
  // no merge launch is needed; several chunks: four waves per chunk
  const int nwv = attn_waves(cut);
  bool tree = false;  // any column that does not see every slot up to its own
  for (int i = 0; i < c.n; ++i) tree = tree || c.vis_base[i] <= c.pos[i];
  if (cut.mfma) {
    ColGroups cg;
    group_columns(c, G, cg);
    const dim3 mg((n_chunks + kMfmaAttnWaves - 1) / kMfmaAttnWaves, s.Hkv, n_set * cg.n);
    const dim3 blk(64 * kMfmaAttnWaves);
    const size_t lds = (size_t)kMfmaAttnWaves * 80 * (s.hd / 8) * sizeof(u32x4);  // per wave a 64-slot V tile and a 16-slot K tile
    if (s.hd == 128 && tree) ES_LAUNCH((attn_mfma_kernel<128, true>), mg, blk, lds, st, a, c, cg, G);
    else if (s.hd == 128) ES_LAUNCH((attn_mfma_kernel<128, false>), mg, blk, lds, st, a, c, cg, G);
    else if (tree) ES_LAUNCH((attn_mfma_kernel<64, true>), mg, blk, lds, st, a, c, cg, G);
    else ES_LAUNCH((attn_mfma_kernel<64, false>), mg, blk, lds, st, a, c, cg, G);
  } else
  DISPATCH_T(s.dtype, {
    if (s.hd == 128 && tree) launch_attn_g<T, 128, true>(G, grid, nwv, st, a, c);
    else if (s.hd == 128) launch_attn_g<T, 128, false>(G, grid, nwv, st, a, c);
    else if (tree) launch_attn_g<T, 64, true>(G, grid, nwv, st, a, c);
    else launch_attn_g<T, 64, false>(G, grid, nwv, st, a, c);
  });
  if (n_chunks > 1) {
    const dim3 mgrid(n_set * c.n, s.Hq);
    DISPATCH_T(s.dtype, {
      if (s.hd == 128) ES_LAUNCH((attn_merge_kernel<T, 128>), mgrid, dim3(128), 0, st, a, c);
      else ES_LAUNCH((attn_merge_kernel<T, 64>), mgrid, dim3(64), 0, st, a, c);
    });
  }
}

}  // namespace es
