// Prefill attention with 64 query rows per wavefront (gfx950).
//
// Same computation as prefill_attn_kernel (Sec. 2.2, Eq. 3-4: the uncached
// suffix rows of a request attend causally over the cached prefix KV gathered
// through the block table and over their own KV), laid out for one wave per
// SIMD:
//
//  * a wave owns two 32-row blocks, so every K row fragment and every
//    transposed V fragment read from LDS feeds two MFMAs, and a workgroup of
//    NW waves shares each K/V tile among NW*64 rows;
//  * the O^T accumulators (2 x d/32 x 16 registers) live in fixed accumulation
//    registers (prism_acc.h), which only the O^T MFMAs touch; the score tiles
//    stay in ordinary registers where the vector ALU works on them;
//  * the software pipeline advances in half tiles of 32 keys (the score
//    buffers of a whole 64-key tile for 64 rows would not fit next to the
//    rest): step u issues the S^T MFMAs of half tile u+1 and the O^T MFMAs of
//    half tile u while the vector ALU does the softmax of half tile u;
//  * K/V tiles of 64 keys still move as whole (page, head) blocks straight
//    into LDS; K has a ring of NSK slots and V of NSV (NSK = NSV or NSV+1), one
//    workgroup barrier per 64-key tile (two steps);
//  * the running maximum is checked per lane against a precomputed bound, so
//    the common path has no cross-lane traffic at all: lanes l and l+32 of a
//    row only talk when some score exceeds the bound (then the maximum is
//    raised and the accumulators are rescaled, as in the 32-row kernel).
#include "prism_acc.h"
#include "prism_device.h"

namespace prism {

template <int D, int NW, int NSK, int NSV>
__global__ __launch_bounds__(NW * 64, 1) void prefill_attn64_kernel(
    const __bf16 *__restrict__ q, const __bf16 *__restrict__ k_pool,
    const __bf16 *__restrict__ v_pool, const int32_t *__restrict__ block_table,
    __bf16 *__restrict__ out, float *__restrict__ partials, const AttnItem *__restrict__ items,
    int Hq, int Hkv, int max_blocks, float scale_log2e) {
  constexpr int RB = 2;                          // 32-row blocks per wave
  constexpr int BN = kTileKeys;                  // keys per copy tile
  constexpr int SK = 32;                         // keys per pipeline step
  constexpr int SUB = BN / SK;                   // steps per tile
  static_assert(NSV >= 2 && (NSK == NSV || NSK == NSV + 1) && NSK >= 3, "ring sizes");
  constexpr int AK = NSK - 1, AV = NSV - 1;      // how many tiles ahead K and V are copied
  constexpr int NT = NW * 64;
  constexpr int BM = NW * 32 * RB;
  constexpr int CPR = D / 8;                     // 16-byte chunks per key row
  constexpr int TILE_BYTES = BN * D * 2;
  constexpr int UNITS = TILE_BYTES / 1024;       // wave-wide 1 KB copies per tile (K or V)
  constexpr int KPU = 1024 / (D * 2);            // keys per copy
  static_assert(UNITS % NW == 0, "copies must divide over the waves");
  constexpr int UPW = UNITS / NW;                // copies per wave per tile (K and V each)
  constexpr int UPP = (kPage * D * 2) / 1024;    // copies per (page, head) block
  constexpr int PPW = UPW > UPP ? UPW / UPP : 1; // pages a wave touches per tile
  constexpr int KK = D / 16;                     // MFMA k-steps over the head dim
  constexpr int DB = D / 32;                     // 32-wide head-dim blocks of O^T
  constexpr int KS = SK / 16;                    // 16-key MFMA k-steps of O^T per step
  static_assert(SUB == 2, "a tile is two steps: the score buffers swap roles an even number of times per tile");

  // LDS: NSK tile slots for K followed by NSV tile slots for V
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  constexpr uint32_t V_RING = (uint32_t)NSK * TILE_BYTES;

  const AttnItem it = items[blockIdx.x];
  if (it.req < 0) return;                        // idle padding entry
  const int G = Hq / Hkv;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31;
  const int hh = lane >> 5;
  const int P = it.prefix, S = it.suffix;
  const int rows_total = S * G;
  const int T = P + S;
  const int nblk = (T + kPage - 1) / kPage;
  const int32_t *bt = block_table + (int64_t)it.req * max_blocks;

  // ---- Q fragments (B operand of S^T): lane holds row l32, dims 16kk+8hh..+7
  const int wrow0 = it.row0 + wave * (32 * RB);
  bf16x8 qf[RB][KK];
  int limit[RB];                                  // last visible key of the lane's row
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int row = wrow0 + rb * 32 + l32;
    const bool valid = row < rows_total;
    const int tok = valid ? row / G : 0;
    const int g = valid ? row % G : 0;
    limit[rb] = valid ? P + tok : -1;
    const __bf16 *qp = q + ((int64_t)(it.q_off + tok) * Hq + it.kv_head * G + g) * D + 8 * hh;
    // rows past the end read the request's first row (a valid address) and are zeroed below
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) qf[rb][kk] = *reinterpret_cast<const bf16x8 *>(qp + 16 * kk);
  }
  // Wave-uniform key bounds: at or below lo_limit no row of the wave is
  // masked, above hi_limit every row is.
  const bool wave_has_rows = wrow0 < rows_total;
  const int first_row = wave_has_rows ? wrow0 : rows_total - 1;
  int last_row = wrow0 + 32 * RB - 1;
  if (last_row > rows_total - 1) last_row = rows_total - 1;
  const int hi_limit = P + last_row / G;

  const int kv_begin = it.kv_begin, kv_end = it.kv_end;
  const int nt = (kv_end - kv_begin + BN - 1) / BN;          // tiles of the workgroup
  int live_steps = 0;                                        // steps this wave computes on
  if (wave_has_rows && hi_limit >= kv_begin) {
    live_steps = (hi_limit - kv_begin) / SK + 1;
    if (live_steps > SUB * nt) live_steps = SUB * nt;
  }
  (void)first_row;

  // O^T block (db, rb) is accumulator tuple db*RB + rb
  static_for<0, DB * RB * 16>([&](auto n_) __attribute__((always_inline)) { acc_write<decltype(n_)::value>(0.f); });
  // m_run: running maximum (raw score units), l_run: running sum, bound: the
  // raw score above which the maximum has to be raised before exponentiating
  float m_run[RB], l_run[RB], bound[RB];
  const float slack = kRescaleThreshold / scale_log2e;
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    m_run[rb] = -1e30f;
    l_run[rb] = 0.f;
    bound[rb] = -1e30f;
  }

  // ---- paged copy: wave w moves units w*UPW .. w*UPW+UPW-1 of a tile; a unit
  // is 1 KB = KPU whole key rows.  Lane l fills LDS slot (row l/CPR, chunk
  // l%CPR) of the unit and therefore fetches chunk (l%CPR) ^ swz(row).
  const int64_t head_off = (int64_t)it.kv_head * (kPage * D * 2);
  const int64_t page_stride = (int64_t)Hkv * (kPage * D * 2);
  uint32_t lane_src[UPW];                         // byte offset inside the (page, head) block
#pragma unroll
  for (int i = 0; i < UPW; ++i) {
    const int key = (wave * UPW + i) * KPU + lane / CPR;   // key inside the tile
    lane_src[i] = (uint32_t)((key % kPage) * (D * 2) + (((lane % CPR) ^ swz<D>(key)) << 4));
  }
  const uint32_t lds_base = lds_address(lds);
  const int wave_blk = (wave * UPW) / UPP;        // first page of a tile this wave copies from
  struct PageIds {
    int32_t p[PPW];
  };
  auto pages_of = [&](int t) -> PageIds {         // page ids of tile t for this wave
    PageIds r;
#pragma unroll
    for (int j = 0; j < PPW; ++j) {
      int blk = (kv_begin + t * BN) / kPage + wave_blk + j;
      if (blk > nblk - 1) blk = nblk - 1;         // never read a table entry past the sequence
      if (blk < 0) blk = 0;
      r.p[j] = bt[blk];
    }
    return r;
  };
  // copy i (0 .. UPW-1) of this wave's share of a tile into a ring slot at
  // byte offset slot_off from the start of LDS
  auto copy_one = [&](const void *pool, uint32_t slot_off, const PageIds &pg, auto it_) __attribute__((always_inline)) {
    constexpr int i = decltype(it_)::value;
    const int u = wave * UPW + i;
    const unsigned char *blk = (const unsigned char *)pool + (int64_t)pg.p[i / UPP] * page_stride + head_off;
    copy16_to_lds(block_resource(blk, kPage * D * 2), lane_src[i], lds_base + slot_off + (uint32_t)(u * 1024));
  };
  auto copy_rows = [&](const void *pool, uint32_t slot_off, const PageIds &pg) __attribute__((always_inline)) {
    static_for<0, UPW>([&](auto i_) __attribute__((always_inline)) { copy_one(pool, slot_off, pg, i_); });
  };
  auto k_slot = [&](int t) -> uint32_t { return (uint32_t)(t % NSK) * TILE_BYTES; };
  // V slots: byte offset from the start of the V ring (the fragment read
  // addresses carry the ring's base, so that every offset fits the 16-bit
  // immediate of an LDS read)
  auto v_slot = [&](int t) -> uint32_t { return (uint32_t)(t % NSV) * TILE_BYTES; };

  const int i16 = lane & 15;
  const int grp = (lane >> 4) & 1;
  // Per-lane LDS addresses of the fragment reads, relative to the start of a
  // tile slot; ring slot, half tile and k-step are constants added on top.
  typedef __attribute__((address_space(3))) const bf16x8 *lds_b128_ptr;
  typedef __attribute__((address_space(3))) s16x4 *lds_tr_ptr;
  uint32_t k_lane[KK];                            // row l32, chunk 2kk+hh
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) k_lane[kk] = lds_base + (uint32_t)lds_off<D>(l32, 2 * kk + hh);
  uint32_t v_lane[DB][2];                         // key 4hh + i16/4 (+8), 4 head dims of block db
#pragma unroll
  for (int db = 0; db < DB; ++db) {
    const int key = 4 * hh + (i16 >> 2);
    const int chunk = 4 * db + 2 * grp + ((i16 & 3) >> 1);
    const int sub = (i16 & 1) << 3;
    v_lane[db][0] = lds_base + V_RING + (uint32_t)(lds_off<D>(key, chunk) + sub);
    v_lane[db][1] = lds_base + V_RING + (uint32_t)(lds_off<D>(key + 8, chunk) + sub);
  }
  // K fragment kk of the 32 keys at byte offset half_off: rows l32, dims 16kk+8hh..+7
  auto k_frag = [&](uint32_t half_off, int kk) -> bf16x8 {
    return *(lds_b128_ptr)(uintptr_t)(k_lane[kk] + half_off);
  };
  // V^T fragment j (0 .. KS*DB-1) of the 32 keys at byte offset half_off: head
  // dims 32db+l32, keys of k-step ks.  Transposing read: within 16 lanes, lane
  // i supplies the address of 4 head dims 4*(i%4).. of key (i/4); it receives
  // 4 keys of head dim i.
  auto v_frag = [&](uint32_t half_off, int j) -> bf16x8 {
    const int ks = j / DB, db = j % DB;
    const uint32_t step_off = half_off + (uint32_t)(ks * 16 * D * 2);
    union {
      s16x4 h[2];
      bf16x8 v;
    } a;
    a.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_ptr)(uintptr_t)(v_lane[db][0] + step_off));
    a.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_ptr)(uintptr_t)(v_lane[db][1] + step_off));
    return a.v;
  };
  auto mask_half = [&](f32x16 (&sx)[RB], int key0) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = key0 + 8 * (r >> 2) + 4 * hh + (r & 3);
        if (key > limit[rb]) sx[rb][r] = -INFINITY;
      }
  };
  // The lane's own maxima of a score half tile against the bound; only when a
  // score exceeds it do the two lanes of a row exchange maxima, raise the
  // running maximum and rescale what has been accumulated.
  auto check_max = [&](const f32x16 (&sx)[RB]) {
    float mx[RB];
    bool grow = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      mx[rb] = sx[rb][0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx[rb] = fmaxf(mx[rb], sx[rb][r]);
      grow |= mx[rb] > bound[rb];
    }
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
      mfma_drain();                               // the accumulators are about to be read
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const float m_new = fmaxf(m_run[rb], max_across_halves(mx[rb]));
        const float alpha = fast_exp2((m_run[rb] - m_new) * scale_log2e);
        m_run[rb] = m_new;
        bound[rb] = m_new + slack;
        l_run[rb] *= alpha;
        static_for<0, DB * 16>([&](auto n_) __attribute__((always_inline)) {
          constexpr int db = decltype(n_)::value / 16, r = decltype(n_)::value % 16;
          if (rb == 0) acc_set<db * RB, r>(acc_get<db * RB, r>() * alpha);
          else acc_set<db * RB + 1, r>(acc_get<db * RB + 1, r>() * alpha);
        });
      }
      __asm__ volatile("s_nop 3");
    }
  };
  // P^T fragment of k-step ks from the scores (exp2, row sums, bf16 rounding)
  auto p_frag = [&](const f32x16 (&sx)[RB], int ks, int rb, float mc) -> bf16x8 {
    bf16x8 pf;
    float sum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float p = fast_exp2(fmaf(sx[rb][8 * ks + e], scale_log2e, -mc));
      sum += p;
      pf[e] = (__bf16)p;
    }
    l_run[rb] += sum;
    return pf;
  };

  // Scores of one half tile, not overlapped with anything (the first one).
  auto plain_scores = [&](f32x16 (&sx)[RB], uint32_t k_half, int key0) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) sx[rb][r] = 0.f;
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      const bf16x8 a = k_frag(k_half, kk);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        sx[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][kk], sx[rb], 0, 0, 0);
    }
    mask_half(sx, key0);
    check_max(sx);
  };
  // Softmax and O^T update of the current half tile, nothing overlapped (the
  // last step a wave computes).
  auto tail_step = [&](f32x16 (&sc)[RB], uint32_t v_half) {
    float mc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) mc[rb] = m_run[rb] * scale_log2e;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 pf[RB];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) pf[rb] = p_frag(sc, ks, rb, mc[rb]);
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 a = v_frag(v_half, ks * DB + db);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
          if (db == 0 && rb == 0) acc_pv<0>(a, pf[rb]);
          static_for<1, DB * RB>([&](auto t_) __attribute__((always_inline)) {
            if (db * RB + rb == decltype(t_)::value) acc_pv<decltype(t_)::value>(a, pf[rb]);
          });
        }
      }
    }
  };

  // The overlapped step: scores of the next half tile into sn, softmax of the
  // current half tile sc, O^T += V^T P^T.  The work is a chain of chunks - one
  // MFMA each, an LDS fragment read LA fragments ahead of its use every other
  // chunk, and a slice of the exponentials - with the compiler's scheduler
  // fenced between chunks.  COPY selects which of this iteration's copies are
  // issued between the chunks (0 none, 1 the V tile, 2 the K tile).
  constexpr int NFR = KK + KS * DB;               // fragments per step: K rows, then V^T
  constexpr int NCH = NFR * RB;                   // chunks (= MFMAs) per step
  constexpr int NX = 16 * RB;                     // score elements per lane per step
  constexpr int LA = 3;
  constexpr int CSPAN = (KK + (KS - 1) * DB) * RB;   // chunks over which the exponentials spread
  PageIds pg_v, pg_k;                             // page ids of the tiles copied next
  // Ring of K / V^T fragments in flight.  It lives across steps: a step starts
  // with its first LA fragments already on their way, requested by the step
  // before it, so that the matrix pipe does not drain at every step boundary
  // while a wave waits for LDS.
  bf16x8 frag[LA + 1];
  static_assert(NFR % (LA + 1) == 0, "a step's fragments fill the ring a whole number of times");
  auto prefetch_first = [&](uint32_t k_half) {    // fragments 0 .. LA-1 of the step that reads k_half
#pragma unroll
    for (int i = 0; i < LA; ++i) frag[i] = k_frag(k_half, i);
  };
  // k_after: where the step after this one finds its K rows (HAS_AFTER says whether there is one)
  auto step = [&](f32x16 (&sc)[RB], f32x16 (&sn)[RB], uint32_t k_next, uint32_t v_cur, int next_key0,
                  auto mask_tag, auto copy_tag, uint32_t copy_slot, auto after_tag,
                  uint32_t k_after) __attribute__((always_inline)) {
    constexpr int COPY = decltype(copy_tag)::value;
    constexpr bool HAS_AFTER = decltype(after_tag)::value;
    float mc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) mc[rb] = m_run[rb] * scale_log2e;
    float sum_even[RB], sum_odd[RB];              // two chains per row: no add waits on the one before it
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) sum_even[rb] = sum_odd[rb] = 0.f;
    bf16x8 pf[KS][RB];                            // P^T fragments, one per 16-key k-step and row block
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) sn[rb][r] = 0.f;
    auto fetch = [&](int i) {                     // fragment i of the chain: K, then V^T, then the next step's K
      if (i < KK) frag[i % (LA + 1)] = k_frag(k_next, i);
      else if (i < NFR) frag[i % (LA + 1)] = v_frag(v_cur, i - KK);
      else if (HAS_AFTER) frag[i % (LA + 1)] = k_frag(k_after, i - NFR);
    };
    // Softmax of the current half tile as a three-stage pipeline over the
    // chunks, walked in the order the O^T MFMAs consume the elements (k-step,
    // row block, key): element x has its exponent argument formed in chunk
    // home(x)-1, exp2 taken in chunk home(x), and is rounded to bf16 (two at a
    // time) and added to the row sum in chunk home(x)+1.
    auto home = [](int x) { return 1 + (x * (CSPAN - 2)) / NX; };
    auto softmax_slice = [&](int c) {
#pragma unroll
      for (int x = 0; x < NX; ++x) {
        const int ks = x / (8 * RB), rb = (x / 8) % RB, e8 = x % 8;
        const int e = 8 * ks + e8;
        if (home(x) == c + 1) sc[rb][e] = fmaf(sc[rb][e], scale_log2e, -mc[rb]);
        if (home(x) == c) sc[rb][e] = fast_exp2(sc[rb][e]);
        if ((x & 1) && home(x) == c - 1) {
          bf16x2 pk;
          pk[0] = (__bf16)sc[rb][e - 1];
          pk[1] = (__bf16)sc[rb][e];
          sum_even[rb] += sc[rb][e - 1];
          sum_odd[rb] += sc[rb][e];
          pf[ks][rb][e8 - 1] = pk[0];
          pf[ks][rb][e8] = pk[1];
        }
      }
    };
    constexpr int CSTRIDE = NCH / UPW;            // one copy every CSTRIDE chunks
    auto mid_copy = [&](int c) __attribute__((always_inline)) {
      if constexpr (COPY != 0) {
        static_for<0, UPW>([&](auto kt) __attribute__((always_inline)) {
          constexpr int k = decltype(kt)::value;
          if (c == k * CSTRIDE + 1) {
            if constexpr (COPY == 1) copy_one(v_pool, copy_slot, pg_v, kt);
            else copy_one(k_pool, copy_slot, pg_k, kt);
          }
        });
      }
    };
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, NCH>([&](auto ct_) __attribute__((always_inline)) {
      constexpr int c = decltype(ct_)::value;
      constexpr int f = c / RB, rb = c % RB;      // fragment and row block of this chunk's MFMA
      if constexpr (rb == 0) fetch(f + LA);
      if constexpr (f < KK) {
        sn[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[f % (LA + 1)], qf[rb][f], sn[rb], 0, 0, 0);
      } else {
        constexpr int j = f - KK;
        acc_pv<(j % DB) * RB + rb>(frag[f % (LA + 1)], pf[j / DB][rb]);
      }
      softmax_slice(c);
      mid_copy(c);
      if (c < NCH - DB * RB) __builtin_amdgcn_sched_barrier(0);
    });
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) l_run[rb] += sum_even[rb] + sum_odd[rb];
    if (decltype(mask_tag)::value) mask_half(sn, next_key0);
    check_max(sn);
  };

  // ---- main loop.  Copies are issued in the fixed order K0 V0 K1 V1 ... and
  // complete in that order.  Iteration t (tile t) reads V of tile t, the
  // second half of K of tile t and the first half of K of tile t+1; it issues
  // the copies of K of tile t+AK and V of tile t+AV (the earlier of the two in
  // the fixed order first) into the slots that iteration t-1 finished with.
  // So at its start "K of t+1 has landed" is a bound on the copies still
  // pending.  Copies past the end of the key range read the (clamped) last
  // page into a free slot and are never used.
  constexpr bool V_FIRST = AK == AV + 1;          // this iteration's V copy precedes its K copy
  constexpr int PENDING_OK = (V_FIRST ? 2 * (AV - 1) : 2 * (AK - 2) + 1) * UPW;
  static_assert((AK + AV + 1) * UPW <= 63, "pending copies must fit the vmcnt counter");
  auto wait_pending = [&](auto n_tag) {
    constexpr int n = decltype(n_tag)::value;
    __builtin_amdgcn_s_waitcnt(0x0F70 | (n & 15) | ((n >> 4) << 14));   // vmcnt(n) only
  };
  f32x16 s_a[RB], s_b[RB];
  PageIds pg_v_next, pg_k_next;                   // ... and of the tiles copied in the iteration after
  if (nt > 0) {
    // K of tile 0 first, and wait for it together with the Q rows loaded
    // above: from here on the only loads in flight are the copies, which the
    // kernel counts itself.
    copy_rows(k_pool, k_slot(0), pages_of(0));
  }
  wait_pending(std::integral_constant<int, 0>{});
  // The Q rows have arrived.  Passing them through an empty statement makes
  // that known to the compiler, which cannot count the copies: otherwise it
  // waits for every outstanding load, copies included, at the first MFMA of
  // each iteration.
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      __asm__ volatile("" : "+v"(qf[rb][kk]));
      if (limit[rb] < 0) qf[rb][kk] = bf16x8{};
    }
  if (nt > 0) {
    {
      const PageIds pg = pages_of(0);
      if (0 < AV) copy_rows(v_pool, V_RING + v_slot(0), pg);
    }
#pragma unroll
    for (int j = 1; j < AK; ++j) {
      const PageIds pg = pages_of(j);
      copy_rows(k_pool, k_slot(j), pg);
      if (j < AV) copy_rows(v_pool, V_RING + v_slot(j), pg);
    }
    pg_v = pages_of(AV);
    pg_k = pages_of(AK);
    pg_v_next = pages_of(AV + 1);
    pg_k_next = pages_of(AK + 1);
    __syncthreads();
    if (live_steps > 0) {
      plain_scores(s_a, k_slot(0), kv_begin);
      if (live_steps > 1) prefetch_first(k_slot(0) + (uint32_t)(SK * D * 2));   // step 0 reads the second half
    }
  }
  auto arrive = [&]() {
    wait_pending(std::integral_constant<int, PENDING_OK>{});   // this wave's part has landed
    __syncthreads();                              // everyone's has; the previous iteration is over
  };
  // after iteration t: the ids for iteration t+1's copies were loaded an
  // iteration ago; start loading those of iteration t+2
  auto next_pages = [&](int t) {
    pg_v = pg_v_next;
    pg_k = pg_k_next;
    pg_v_next = pages_of(t + 2 + AV);
    pg_k_next = pages_of(t + 2 + AK);
  };
  // Tiles 0 .. n_fast-1: every score computed while they are processed (up to
  // the first half of the following tile) is visible to every row of the
  // workgroup, so no mask is needed and every wave with rows is busy in every
  // step.  They run lcm(NSK, NSV) tiles per trip with the ring slots fixed in
  // the code, so every LDS address is a register plus an immediate.
  int n_fast = 0;
  {
    const int blk_limit = P + it.row0 / G;        // last key visible to the workgroup's first row
    const int span = blk_limit - kv_begin - (BN + SK - 1);
    if (span >= 0) n_fast = span / BN + 1;
    if (n_fast > nt - 1) n_fast = nt - 1;
    if (n_fast < 0) n_fast = 0;
  }
  constexpr int UNROLL = NSK == NSV ? NSK : NSK * NSV;   // equal or consecutive: the least common multiple
  auto fast_iteration = [&](int t, auto j_tag) __attribute__((always_inline)) {
    constexpr int j = decltype(j_tag)::value;     // t % UNROLL
    constexpr uint32_t k_cur = (uint32_t)(j % NSK) * TILE_BYTES;
    constexpr uint32_t k_nxt = (uint32_t)((j + 1) % NSK) * TILE_BYTES;
    constexpr uint32_t v_cur = (uint32_t)(j % NSV) * TILE_BYTES;
    constexpr uint32_t v_new = V_RING + (uint32_t)((j + AV) % NSV) * TILE_BYTES;
    constexpr uint32_t k_new = (uint32_t)((j + AK) % NSK) * TILE_BYTES;
    constexpr uint32_t HALF = (uint32_t)SK * D * 2;
    using CopyV = std::integral_constant<int, 1>;
    using CopyK = std::integral_constant<int, 2>;
    arrive();
    if (wave_has_rows) {
      // the step after the first reads the start of K of tile t+1, the one
      // after the second (in the next iteration) its second half
      if constexpr (V_FIRST) {
        step(s_a, s_b, k_cur + HALF, v_cur, 0, std::false_type{}, CopyV{}, v_new, std::true_type{}, k_nxt);
        step(s_b, s_a, k_nxt, v_cur + HALF, 0, std::false_type{}, CopyK{}, k_new, std::true_type{}, k_nxt + HALF);
      } else {
        step(s_a, s_b, k_cur + HALF, v_cur, 0, std::false_type{}, CopyK{}, k_new, std::true_type{}, k_nxt);
        step(s_b, s_a, k_nxt, v_cur + HALF, 0, std::false_type{}, CopyV{}, v_new, std::true_type{}, k_nxt + HALF);
      }
    } else if constexpr (V_FIRST) {               // a wave without rows only copies
      copy_rows(v_pool, v_new, pg_v);
      copy_rows(k_pool, k_new, pg_k);
    } else {
      copy_rows(k_pool, k_new, pg_k);
      copy_rows(v_pool, v_new, pg_v);
    }
    next_pages(t);
  };
  int t = 0;
  for (; t + UNROLL <= n_fast; t += UNROLL)
    static_for<0, UNROLL>([&](auto j_) __attribute__((always_inline)) { fast_iteration(t + decltype(j_)::value, j_); });
  // The remaining tiles (the causal diagonal, a short key range, the last
  // tile): the same overlapped step with the mask applied to the new scores
  // and ring slots chosen at run time; a wave stops computing after the last
  // step that any of its rows can see.
  for (; t < nt; ++t) {
    arrive();
    if constexpr (V_FIRST) {
      copy_rows(v_pool, V_RING + v_slot(t + AV), pg_v);
      copy_rows(k_pool, k_slot(t + AK), pg_k);
    } else {
      copy_rows(k_pool, k_slot(t + AK), pg_k);
      copy_rows(v_pool, V_RING + v_slot(t + AV), pg_v);
    }
    next_pages(t);
    if (t == nt - 1 && kv_begin + nt * BN > T) {
      // Slots past the end of the sequence hold whatever the pool held: clear
      // those V rows so that 0 * garbage cannot poison the products.
      const uint32_t vs = V_RING + v_slot(t);
      for (int c = tid; c < BN * CPR; c += NT)
        if (kv_begin + t * BN + c / CPR >= T)
          *reinterpret_cast<u32x4 *>(lds + vs + c * 16) = u32x4{0u, 0u, 0u, 0u};
      __syncthreads();
    }
#pragma unroll
    for (int h = 0; h < SUB; ++h) {
      const int u = t * SUB + h;
      const uint32_t v_half = v_slot(t) + (uint32_t)(h * SK * D * 2);
      if (u + 1 < live_steps) {
        // half tile u+1 is the second half of tile t (h = 0) or the start of
        // tile t+1 (h = 1); half tile u+2 the start of tile t+1 or its second half
        const uint32_t k_half = h == 0 ? k_slot(t) + (uint32_t)(SK * D * 2) : k_slot(t + 1);
        const uint32_t k_after = h == 0 ? k_slot(t + 1) : k_slot(t + 1) + (uint32_t)(SK * D * 2);
        if (u + 2 < live_steps)
          step(s_a, s_b, k_half, v_half, kv_begin + (u + 1) * SK, std::true_type{},
               std::integral_constant<int, 0>{}, 0u, std::true_type{}, k_after);
        else
          step(s_a, s_b, k_half, v_half, kv_begin + (u + 1) * SK, std::true_type{},
               std::integral_constant<int, 0>{}, 0u, std::false_type{}, 0u);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) s_a[rb] = s_b[rb];
      } else if (u < live_steps) {
        tail_step(s_a, v_half);
      }
    }
  }
  wait_pending(std::integral_constant<int, 0>{});   // let the unused trailing copies drain
  mfma_drain();

  // ---- epilogue
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int row = wrow0 + rb * 32 + l32;
    const float l_tot = sum_across_halves(l_run[rb]);
    float o_val[DB][16];                          // this row block's O^T columns out of the accumulators
    static_for<0, DB * 16>([&](auto n_) __attribute__((always_inline)) {
      constexpr int db = decltype(n_)::value / 16, r = decltype(n_)::value % 16;
      o_val[db][r] = rb == 0 ? acc_get<db * RB, r>() : acc_get<db * RB + 1, r>();
    });
    if (row >= rows_total) continue;
    if (it.part_slot < 0) {
      const float inv = 1.0f / l_tot;
      const int tok = row / G, g = row % G;
      __bf16 *op = out + ((int64_t)(it.q_off + tok) * Hq + it.kv_head * G + g) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          bf16x4 o4;
#pragma unroll
          for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(o_val[db][4 * g4 + e] * inv);
          *reinterpret_cast<bf16x4 *>(op + 32 * db + 8 * g4 + 4 * hh) = o4;
        }
    } else {
      float *slot = partials + (size_t)it.part_slot * ((size_t)BM * (D + 2));
      const int lr = row - it.row0;
      float *po = slot + (size_t)lr * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          float4 o4;
          o4.x = o_val[db][4 * g4 + 0];
          o4.y = o_val[db][4 * g4 + 1];
          o4.z = o_val[db][4 * g4 + 2];
          o4.w = o_val[db][4 * g4 + 3];
          *reinterpret_cast<float4 *>(po + 32 * db + 8 * g4 + 4 * hh) = o4;
        }
      if (hh == 0) {
        slot[(size_t)BM * D + lr] = m_run[rb];
        slot[(size_t)BM * D + BM + lr] = l_tot;
      }
    }
  }
}

template <int D, int NW, int NSK, int NSV>
static int launch_attn64_t(const LaunchParams &p, hipStream_t st) {
  constexpr size_t lds_bytes = (size_t)(NSK + NSV) * kTileKeys * D * 2;
  auto kernel = prefill_attn64_kernel<D, NW, NSK, NSV>;
  static const hipError_t attr = hipFuncSetAttribute(
      (const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (attr != hipSuccess) return (int)attr;
  return launch_kernel(kernel, dim3((unsigned)p.num_items), dim3(NW * 64), lds_bytes, st,
                       (const __bf16 *)p.q, (const __bf16 *)p.k_pool, (const __bf16 *)p.v_pool,
                       p.block_table, (__bf16 *)p.out, p.partials, p.items, p.Hq, p.Hkv, p.max_blocks,
                       p.scale_log2e);
}

// 128 rows: two waves, two workgroups per compute unit, K ring of 3 and V ring
// of 2 tiles (80 KB at d = 128, so that two fit in the 160 KB of LDS).
// 256 rows: four waves, one workgroup per compute unit, rings of 4 and 4
// tiles (128 KB at d = 128).
int launch_attention64(const LaunchParams &p, void *stream) {
  if (p.num_items == 0) return 0;
  hipStream_t st = (hipStream_t)stream;
  if (p.d == 128) {
    if (p.tile_rows == 128) return launch_attn64_t<128, 2, 3, 2>(p, st);
    return launch_attn64_t<128, 4, 4, 4>(p, st);
  }
  if (p.tile_rows == 128) return launch_attn64_t<64, 2, 3, 2>(p, st);
  return launch_attn64_t<64, 4, 4, 4>(p, st);
}

}  // namespace prism
