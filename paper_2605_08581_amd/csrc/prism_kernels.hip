// HIP kernels for gfx950 (CDNA4): paged KV append, paged flash-style prefill
// attention with bf16 MFMA, and the split-KV merge.
//
// What is computed follows the paper's statement of prefix reuse (Sec. 2.2,
// Eq. 3-4): the uncached suffix rows of each request attend causally over the
// cached prefix KV (gathered through the block table) and over their own KV.
#include "prism_device.h"

namespace prism {

// --------------------------------------------------------------------------
// Paged KV append.  One thread moves 16 bytes of K and 16 bytes of V.  Block
// row y of the grid serves request req0 + y of the chunk; its prefix, suffix
// and source offset arrive in the kernel arguments.
// --------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void kv_append_kernel(
    const u32x4 *__restrict__ k_src, const u32x4 *__restrict__ v_src, u32x4 *__restrict__ k_pool,
    u32x4 *__restrict__ v_pool, const int32_t *__restrict__ block_table, const AppendChunk chunk,
    int Hkv, int max_blocks) {
  constexpr int CH = D / 8;                       // 16-byte chunks per (token, head) row
  const int y = blockIdx.y;
  const int S = chunk.suffix[y], P = chunk.prefix[y];
  const int per_tok = Hkv * CH;
  const int total = S * per_tok;                  // < 2^31: checked at plan creation
  const int32_t *bt = block_table + (int64_t)(chunk.req0 + y) * max_blocks;
  const int64_t src0 = (int64_t)chunk.q_off[y] * per_tok;
  for (int c = blockIdx.x * blockDim.x + threadIdx.x; c < total; c += gridDim.x * blockDim.x) {
    const int tok = c / per_tok;
    const int rem = c - tok * per_tok;
    const int h = rem / CH, ch = rem % CH;
    const int pos = P + tok;
    const int32_t page = bt[pos / kPage];
    const int64_t dst = (((int64_t)page * Hkv + h) * kPage + (pos % kPage)) * CH + ch;
    k_pool[dst] = k_src[src0 + c];
    v_pool[dst] = v_src[src0 + c];
  }
}

int launch_append(const void *k_src, const void *v_src, void *k_pool, void *v_pool,
                  const int32_t *block_table, const AppendChunk &chunk, int max_suffix, int Hkv, int d,
                  int max_blocks, void *stream) {
  if (chunk.nreq == 0 || max_suffix == 0) return 0;
  const int64_t longest = (int64_t)max_suffix * Hkv * (d / 8);
  int64_t bx = (longest + 255) / 256;
  if (bx > 1024) bx = 1024;                       // longer requests loop
  const dim3 grid((unsigned)bx, (unsigned)chunk.nreq), block(256);
  hipStream_t st = (hipStream_t)stream;
  if (d == 128)
    return launch_kernel(kv_append_kernel<128>, grid, block, 0, st, (const u32x4 *)k_src, (const u32x4 *)v_src,
                         (u32x4 *)k_pool, (u32x4 *)v_pool, block_table, chunk, Hkv, max_blocks);
  return launch_kernel(kv_append_kernel<64>, grid, block, 0, st, (const u32x4 *)k_src, (const u32x4 *)v_src,
                       (u32x4 *)k_pool, (u32x4 *)v_pool, block_table, chunk, Hkv, max_blocks);
}

// --------------------------------------------------------------------------
// Prefill attention.
//
// A workgroup of NW waves owns NW*32*RB packed query rows of one (request, kv
// head) and walks the key range in tiles of 64 keys (four 16-token pages).
// K and V rows are copied from the paged pool straight into LDS
// (global_load_lds, 16 bytes per lane, no staging registers); K and V each
// have a two-slot ring, and there is one workgroup barrier per tile.
//
// Per wave the products are taken transposed so that no value ever has to move
// between lanes except one exchange for the row maximum:
//   S^T = K Q^T   (MFMA 32x32x16: A = K rows from LDS, B = Q rows in registers)
//   O^T = V^T P^T (A = V read transposed from LDS, B = P^T straight from the
//                  S^T accumulators, rounded to bf16)
// In the 32x32 accumulator layout lane l holds column l%32 (a query row) and
// rows 8*(r/4) + 4*(l/32) + r%4, r = 0..15 (keys for S^T, head dims for O^T),
// so the running max, the running sum and the rescale factor of a query row
// are per-lane scalars.
//
// The loop is software pipelined inside each wave: iteration t issues the
// S^T MFMAs of tile t+1 and the O^T MFMAs of tile t while the vector ALU does
// the softmax of tile t, so the matrix pipe and the vector pipe of a SIMD work
// at the same time instead of taking turns.
//
// LDS rows are d bf16 wide, 16-byte chunks XOR-swizzled by the key index so
// that both the row reads (K) and the transposing reads (V) spread over banks.
// A direct-to-LDS load writes lane l's 16 bytes at (wave-uniform base) + 16*l,
// so the swizzle is applied on the global side: lane l fetches the chunk that
// belongs in the slot it will fill.
//
// The running maximum is only raised when some row's tile maximum exceeds it
// by more than 2^8 in the exponent domain: probabilities then stay below 256,
// the final division by the row sum cancels the offset exactly, and the
// accumulator rescale is skipped on almost every tile.
// --------------------------------------------------------------------------

template <int D, int RB, int NW, int WPE, int NS>
__global__ __launch_bounds__(NW * 64, WPE) void prefill_attn_kernel(
    const __bf16 *__restrict__ q, const __bf16 *__restrict__ k_pool,
    const __bf16 *__restrict__ v_pool, const int32_t *__restrict__ block_table,
    __bf16 *__restrict__ out, float *__restrict__ partials, const AttnItem *__restrict__ items,
    int Hq, int Hkv, int max_blocks, float scale_log2e) {
  constexpr int BN = kTileKeys;
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
  constexpr int KB = BN / 32;                    // 32-key blocks per tile
  constexpr int KS = BN / 16;                    // 16-key MFMA k-steps of O^T per tile

  // LDS: a ring of NS tile slots for K followed by a ring of NS slots for V
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  static_assert(NS >= 2, "each ring needs the slot in use and one being filled");
  // byte offsets of the ring slots that hold tile t
  auto k_slot = [&](int t) -> uint32_t { return (uint32_t)(t % NS) * TILE_BYTES; };
  auto v_slot = [&](int t) -> uint32_t { return (uint32_t)(NS + t % NS) * TILE_BYTES; };

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
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
      bf16x8 v = {};
      if (valid) v = *reinterpret_cast<const bf16x8 *>(qp + 16 * kk);
      qf[rb][kk] = v;
    }
  }
  // Wave-uniform key bounds: at or below lo_limit no row of the wave is
  // masked, above hi_limit every row is.
  const int first_row = wrow0 < rows_total ? wrow0 : rows_total - 1;
  int last_row = wrow0 + 32 * RB - 1;
  if (last_row > rows_total - 1) last_row = rows_total - 1;
  const int lo_limit = P + first_row / G;
  const int hi_limit = P + last_row / G;

  const int kv_begin = it.kv_begin, kv_end = it.kv_end;
  const int nt = (kv_end - kv_begin + BN - 1) / BN;          // tiles of the workgroup
  int my_nt = 0;                                             // tiles this wave computes on
  if (wrow0 < rows_total && hi_limit >= kv_begin) {
    my_nt = (hi_limit - kv_begin) / BN + 1;
    if (my_nt > nt) my_nt = nt;
  }

  f32x16 oacc[DB][RB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[db][rb][r] = 0.f;
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
  // is 1 KB = KPU whole key rows, and consecutive units stay inside one
  // (page, head) block as long as possible so a wave needs few page ids.
  // Lane l fills LDS slot (row l/CPR, chunk l%CPR) of the unit and therefore
  // fetches chunk (l%CPR) ^ swz(row).
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
      r.p[j] = bt[blk];
    }
    return r;
  };
  auto copy_rows = [&](const void *pool, int which, int slot, const PageIds &pg) {
#pragma unroll
    for (int i = 0; i < UPW; ++i) {
      const int u = wave * UPW + i;
      const unsigned char *blk =                                      // wave-uniform
          (const unsigned char *)pool + (int64_t)pg.p[i / UPP] * page_stride + head_off;
      copy16_to_lds(block_resource(blk, kPage * D * 2), lane_src[i],
                    lds_base + (uint32_t)((which * NS + slot) * TILE_BYTES + u * 1024));
    }
  };

  PageIds pg_v, pg_k;                             // page ids of tiles t+NS-1 and t+NS
  // copy i (0 .. UPW-1) of this wave's share of a tile, as one instruction
  auto copy_one = [&](const void *pool, int which, int slot, const PageIds &pg, auto it_) __attribute__((always_inline)) {
    constexpr int i = decltype(it_)::value;
    const int u = wave * UPW + i;
    const unsigned char *blk = (const unsigned char *)pool + (int64_t)pg.p[i / UPP] * page_stride + head_off;
    copy16_to_lds(block_resource(blk, kPage * D * 2), lane_src[i],
                  lds_base + (uint32_t)((which * NS + slot) * TILE_BYTES + u * 1024));
  };
  const int i16 = lane & 15;
  const int grp = (lane >> 4) & 1;

  // Per-lane LDS addresses of the fragment reads, relative to the start of a
  // tile slot; everything else (ring slot, 32-key block, k-step) is a constant
  // added on top, so a read is one address register plus an immediate.
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
    v_lane[db][0] = lds_base + (uint32_t)(lds_off<D>(key, chunk) + sub);
    v_lane[db][1] = lds_base + (uint32_t)(lds_off<D>(key + 8, chunk) + sub);
  }
  // K fragment i (0 .. KB*KK-1) of the tile in K ring slot at byte offset
  // slot_off: rows kb*32+l32, dims 16kk+8hh..+7
  auto k_frag = [&](uint32_t slot_off, int i) -> bf16x8 {
    return *(lds_b128_ptr)(uintptr_t)(k_lane[i % KK] + slot_off + (uint32_t)((i / KK) * 32 * D * 2));
  };
  // V^T fragment j (0 .. KS*DB-1): head dims 32db+l32, keys of k-step ks.
  // Transposing read: within 16 lanes, lane i supplies the address of 4 head
  // dims 4*(i%4).. of key (i/4); it receives 4 keys of head dim i.
  auto v_frag = [&](uint32_t slot_off, int j) -> bf16x8 {
    const int ks = j / DB, db = j % DB;
    const uint32_t step_off = slot_off + (uint32_t)(ks * 16 * D * 2);
    union {
      s16x4 h[2];
      bf16x8 v;
    } a;
    a.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_ptr)(uintptr_t)(v_lane[db][0] + step_off));
    a.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_tr_ptr)(uintptr_t)(v_lane[db][1] + step_off));
    return a.v;
  };
  auto mask_tile = [&](f32x16 (&sx)[KB][RB], int key0) {
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = key0 + kb * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
          if (key > limit[rb]) sx[kb][rb][r] = -INFINITY;
        }
  };
  // The lane's own maximum of a score tile against a precomputed bound (the
  // running maximum plus the slack): no cross-lane traffic on the common path.
  // Only when some score of the wave exceeds its bound do the two lanes of a
  // row exchange maxima, raise the running maximum and rescale what has been
  // accumulated.
  auto raise_max = [&](const f32x16 (&sx)[KB][RB]) {
    float mx[RB];
    bool grow = false;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      mx[rb] = sx[0][rb][0];
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx[rb] = fmaxf(mx[rb], sx[kb][rb][r]);
      grow |= mx[rb] > bound[rb];
    }
    if (__builtin_amdgcn_ballot_w64(grow) != 0) {
      if constexpr (RB > 1) mfma_drain();
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) {
        const float m_new = fmaxf(m_run[rb], max_across_halves(mx[rb]));
        bound[rb] = m_new + slack;
        const float alpha = fast_exp2((m_run[rb] - m_new) * scale_log2e);
        m_run[rb] = m_new;
        l_run[rb] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[db][rb][r] *= alpha;
      }
      if constexpr (RB > 1) __asm__ volatile("s_nop 1");
    }
  };
  // P^T fragment of k-step ks from the scores (exp2, row sums, bf16 rounding)
  auto p_frag = [&](const f32x16 (&sx)[KB][RB], int ks, int rb, float mc) -> bf16x8 {
    bf16x8 pf;
    float sum = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float p = fast_exp2(fmaf(sx[ks >> 1][rb][8 * (ks & 1) + e], scale_log2e, -mc));
      sum += p;                                   // the fp32 exponentials, as in the overlapped step
      pf[e] = (__bf16)p;
    }
    l_run[rb] += sum;
    return pf;
  };

  // Scores of one tile, not overlapped with anything (first tile, and tiles
  // that need the causal mask).
  auto plain_scores = [&](f32x16 (&sx)[KB][RB], uint32_t k_lds, int key0, bool masked) {
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) sx[kb][rb][r] = 0.f;
#pragma unroll
    for (int i = 0; i < KB * KK; ++i) {
      const bf16x8 a = k_frag(k_lds, i);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
        sx[i / KK][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][i % KK], sx[i / KK][rb], 0, 0, 0);
    }
    if (masked) mask_tile(sx, key0);
    raise_max(sx);
  };
  // Softmax and O^T update of the current tile, nothing overlapped (tiles on
  // the causal diagonal and the last tile).
  auto tail_step = [&](f32x16 (&sc)[KB][RB], uint32_t v_cur) {
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
        const bf16x8 a = v_frag(v_cur, ks * DB + db);
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) pv_mfma<(RB > 1)>(oacc[db][rb], a, pf[rb]);
      }
    }
  };

  // The overlapped step: scores of the next (unmasked) tile into sn, softmax
  // of the current tile sc, O^T += V^T P^T.  The work is laid out as a chain
  // of chunks - one MFMA, one LDS fragment read three chunks ahead of its
  // use, and a slice of the exponentials - and the compiler's scheduler is
  // fenced between chunks, so the matrix pipe always has an MFMA queued while
  // the vector ALU works through the softmax.  When VSLOT/KSLOT name ring
  // slots (>= 0), this wave's copies of the tiles that go into them are issued
  // one at a time between the first chunks (every other one), instead of in a
  // burst before the step: a copy instruction that finds the load queue full
  // then holds up one wave for a moment rather than every wave of the
  // workgroup at once, and the data still has most of an iteration to arrive.
  constexpr int NQK = KB * KK;                    // K fragments per tile (one S^T MFMA each per row block)
  constexpr int NPV = KS * DB;                    // V^T fragments per tile (one O^T MFMA each per row block)
  constexpr int NEL = KB * 16;                    // score elements per lane per row block
  constexpr int LA = 3;                           // fragment reads run this many fragments ahead
  constexpr int NCH = (NQK + NPV) * RB;           // chunks (= MFMAs) per step
  constexpr int CSPAN = (NQK + (KS - 1) * DB) * RB;   // chunks over which the exponentials spread
  auto step = [&](f32x16 (&sc)[KB][RB], f32x16 (&sn)[KB][RB], uint32_t k_next, uint32_t v_cur,
                  int next_key0, auto mask_tag, auto vslot_tag, auto kslot_tag) __attribute__((always_inline)) {
    constexpr int VSLOT = decltype(vslot_tag)::value, KSLOT = decltype(kslot_tag)::value;
    constexpr int NC = 2 * UPW;
    constexpr int STRIDE = 2 * NC <= NCH ? 2 : 1;   // every other chunk from the start of the step
    float mc[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) mc[rb] = m_run[rb] * scale_log2e;
    float sum_even[RB], sum_odd[RB];              // two chains per row: no add waits on the one before it
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) sum_even[rb] = sum_odd[rb] = 0.f;
    bf16x8 frag[LA + 1];                          // ring of K / V^T fragments in flight
    bf16x8 pf[KS][RB];                            // P^T fragments, one per 16-key k-step and row block
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) sn[kb][rb][r] = 0.f;
    auto fetch = [&](int i) {                     // fragment i of the chain: K first, then V^T
      if (i < NQK) frag[i % (LA + 1)] = k_frag(k_next, i);
      else if (i < NQK + NPV) frag[i % (LA + 1)] = v_frag(v_cur, i - NQK);
    };
    // Softmax of the current tile, spread over the chunks as a three-stage
    // pipeline so that no chunk waits on its own results.  The elements are
    // walked in the order the O^T MFMAs consume them (k-step, row block, key);
    // element x has its exponent argument formed in chunk home(x)-1, exp2
    // taken in chunk home(x), and is rounded to bf16 (two at a time) and added
    // to the row sum in chunk home(x)+1.  The row sum adds the fp32
    // exponentials (before the rounding): plain adds on two alternating chains
    // measured 2 % faster over the whole kernel than a packed dot product of
    // the rounded pairs, and the difference to the rounded sum is far inside
    // the tolerance.
    constexpr int NX = NEL * RB;
    auto home = [](int x) { return 1 + (x * (CSPAN - 2)) / NX; };
    auto softmax_slice = [&](int c) {
#pragma unroll
      for (int x = 0; x < NX; ++x) {
        const int ks = x / (8 * RB), rb = (x / 8) % RB, e8 = x % 8;
        const int e = 8 * ks + e8;                // element of the row block's tile column
        if (home(x) == c + 1) sc[e / 16][rb][e % 16] = fmaf(sc[e / 16][rb][e % 16], scale_log2e, -mc[rb]);
        if (home(x) == c) sc[e / 16][rb][e % 16] = fast_exp2(sc[e / 16][rb][e % 16]);
        if ((x & 1) && home(x) == c - 1) {
          bf16x2 pk;
          pk[0] = (__bf16)sc[e / 16][rb][(e - 1) % 16];
          pk[1] = (__bf16)sc[e / 16][rb][e % 16];
          sum_even[rb] += sc[e / 16][rb][(e - 1) % 16];
          sum_odd[rb] += sc[e / 16][rb][e % 16];
          pf[ks][rb][e8 - 1] = pk[0];
          pf[ks][rb][e8] = pk[1];
        }
      }
    };
    auto mid_copy = [&](int c) __attribute__((always_inline)) {   // V copies first, then K
      if (VSLOT < 0) return;
      static_for<0, NC>([&](auto kt) __attribute__((always_inline)) {
        constexpr int k = decltype(kt)::value;
        if (c == k * STRIDE + STRIDE - 1) {
          if constexpr (k < UPW) copy_one(v_pool, 1, VSLOT, pg_v, std::integral_constant<int, k>{});
          else copy_one(k_pool, 0, KSLOT, pg_k, std::integral_constant<int, k - UPW>{});
        }
      });
    };
#pragma unroll
    for (int i = 0; i < LA; ++i) fetch(i);
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, NCH>([&](auto ct_) __attribute__((always_inline)) {
      constexpr int c = decltype(ct_)::value;
      constexpr int f = c / RB, rb = c % RB;      // fragment and row block of this chunk's MFMA
      if constexpr (rb == 0) fetch(f + LA);
      if constexpr (f < NQK) {
        sn[f / KK][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[f % (LA + 1)], qf[rb][f % KK],
                                                                 sn[f / KK][rb], 0, 0, 0);
      } else {
        constexpr int j = f - NQK;
        pv_mfma<(RB > 1)>(oacc[j % DB][rb], frag[f % (LA + 1)], pf[j / DB][rb]);
      }
      softmax_slice(c);
      mid_copy(c);
      if (c < NCH - DB * RB) __builtin_amdgcn_sched_barrier(0);
    });
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) l_run[rb] += sum_even[rb] + sum_odd[rb];
    if (decltype(mask_tag)::value) mask_tile(sn, next_key0);   // the next tile touches the diagonal
    raise_max(sn);
  };

  // ---- main loop.  At the start of iteration t the scores of tile t are in
  // registers, K of tile t+1 and V of tile t are in LDS, and the copies of the
  // next NS-2 tiles of each are in flight; the iteration starts the copies of
  // V of tile t+NS-1 and K of tile t+NS into the slots that iteration t-1
  // finished with, and ends with the scores of tile t+1.  Copies are issued in
  // the fixed order K0 V0 K1 V1 ... and complete in that order, so "K of t+1
  // and V of t have landed" is "at most 2(NS-2) tile copies still pending".
  // Copies past the end of the key range read the (clamped) last page into a
  // free slot and are never used: that keeps the pending count uniform.
  constexpr int PENDING_OK = 2 * (NS - 2) * UPW;
  static_assert((2 * NS - 2) * UPW <= 63, "pending copies must fit the vmcnt counter");
  auto wait_pending = [&](auto n_tag) {
    constexpr int n = decltype(n_tag)::value;
    __builtin_amdgcn_s_waitcnt(0x0F70 | (n & 15) | ((n >> 4) << 14));   // vmcnt(n) only
  };
  const bool wave_live = my_nt > 0;
  f32x16 s_a[KB][RB], s_b[KB][RB];
  if (nt > 0) copy_rows(k_pool, 0, 0, pages_of(0));
  if constexpr (NS > 2) {
    // With rings deeper than two slots copies stay in flight across
    // iterations.  The compiler cannot count them (they are inline assembly),
    // so as long as it believes the Q rows loaded above may still be on their
    // way it waits for every outstanding load at the first MFMA of each
    // iteration.  Wait here, once, for Q and K of tile 0, and pass the Q
    // registers through an empty statement so that it knows.
    wait_pending(std::integral_constant<int, 0>{});
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) __asm__ volatile("" : "+v"(qf[rb][kk]));
  }
  if (nt > 0) {
    PageIds pg = pages_of(0);
    copy_rows(v_pool, 1, 0, pg);
    pg = pages_of(1);
#pragma unroll
    for (int j = 1; j < NS - 1; ++j) {
      copy_rows(k_pool, 0, j, pg);
      copy_rows(v_pool, 1, j, pg);
      pg = pages_of(j + 1);
    }
    copy_rows(k_pool, 0, NS - 1, pg);
    pg_v = pg;
    pg_k = pages_of(NS);
    wait_pending(std::integral_constant<int, (2 * NS - 2) * UPW>{});   // K of tile 0 is in
    __syncthreads();
    if (wave_live) plain_scores(s_a, k_slot(0), kv_begin, kv_begin + BN - 1 > lo_limit);
  }
  // j is the tile index modulo NS, known at compile time in the fast loop so
  // that every LDS address there is a register plus an immediate.
  auto issue_copies = [&](int v_ring_slot, int k_ring_slot, int t) {
    copy_rows(v_pool, 1, v_ring_slot, pg_v);
    copy_rows(k_pool, 0, k_ring_slot, pg_k);
    pg_v = pg_k;
    pg_k = pages_of(t + NS + 1);
  };
  auto arrive = [&]() {
    wait_pending(std::integral_constant<int, PENDING_OK>{});   // this wave's part has landed
    __syncthreads();                              // everyone's has; the previous iteration is over
  };
  // Tiles 0 .. n_fast-1 are followed by a tile that no row of the workgroup
  // needs masked.  They run NS per trip with j = t % NS a compile-time value,
  // so that ring slots and the score buffer in use are fixed in the code and
  // every LDS address is a register plus an immediate.
  int n_fast = 0;
  {
    const int blk_limit = P + it.row0 / G;        // last key visible to the workgroup's first row
    if (blk_limit >= kv_begin + 2 * BN - 1) n_fast = (blk_limit + 1 - kv_begin) / BN - 1;
    if (n_fast > nt - 1) n_fast = nt - 1;
    if (n_fast < 0) n_fast = 0;
  }
  auto fast_iteration = [&](int t, auto j_tag) __attribute__((always_inline)) {
    constexpr int j = decltype(j_tag)::value;
    static_assert(NS % 2 == 0, "score buffers alternate with the tile parity");
    constexpr uint32_t k_next = (uint32_t)((j + 1) % NS) * TILE_BYTES;
    constexpr uint32_t v_cur = (uint32_t)(NS + j) * TILE_BYTES;
    arrive();
    if (wave_live) {
      // the step issues this iteration's copies itself, between its chunks
      using VSlot = std::integral_constant<int, (j + NS - 1) % NS>;
      using KSlot = std::integral_constant<int, j>;
      if (j % 2 == 0) step(s_a, s_b, k_next, v_cur, 0, std::false_type{}, VSlot{}, KSlot{});
      else step(s_b, s_a, k_next, v_cur, 0, std::false_type{}, VSlot{}, KSlot{});
      pg_v = pg_k;
      pg_k = pages_of(t + NS + 1);
    } else {
      issue_copies((j + NS - 1) % NS, j, t);      // a wave with no rows left only copies
    }
  };
  static_assert(NS == 2 || NS == 4, "the loop is unrolled for rings of 2 or 4 slots");
  int t = 0;
  for (; t + NS <= n_fast; t += NS) {
    fast_iteration(t, std::integral_constant<int, 0>{});
    fast_iteration(t + 1, std::integral_constant<int, 1>{});
    if (NS > 2) {
      fast_iteration(t + 2, std::integral_constant<int, 2 % NS>{});
      fast_iteration(t + 3, std::integral_constant<int, 3 % NS>{});
    }
  }
  // The tiles up to the causal diagonal (and a few left over from the loop
  // above): the same overlapped step with the causal mask applied to the new
  // scores, ring slots chosen at run time, scores handed back in s_a.  (A wave
  // whose rows end early computes fully masked tiles until the workgroup's key
  // range ends - at most two - and they add exact zeros.)
  for (; t + 1 < nt; ++t) {
    arrive();
    issue_copies((t + NS - 1) % NS, t % NS, t);
    if (wave_live) {
      step(s_a, s_b, k_slot(t + 1), v_slot(t), kv_begin + (t + 1) * BN, std::true_type{},
           std::integral_constant<int, -1>{}, std::integral_constant<int, -1>{});
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) s_a[kb][rb] = s_b[kb][rb];
    }
  }
  if (nt > 0) {                                   // the last tile: softmax and PV only
    const uint32_t v_cur = v_slot(t);
    arrive();
    if (kv_begin + nt * BN > T) {
      // Slots past the end of the sequence hold whatever the pool held: clear
      // those V rows so that 0 * garbage cannot poison the products.
      for (int c = tid; c < BN * CPR; c += NT)
        if (kv_begin + t * BN + c / CPR >= T)
          *reinterpret_cast<u32x4 *>(lds + v_cur + c * 16) = u32x4{0u, 0u, 0u, 0u};
      __syncthreads();
    }
    if (wave_live) tail_step(s_a, v_cur);
  }
  wait_pending(std::integral_constant<int, 0>{});   // let the unused trailing copies drain
  if constexpr (RB > 1) mfma_drain();

  // ---- epilogue
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int row = wrow0 + rb * 32 + l32;
    const float l_tot = sum_across_halves(l_run[rb]);
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
          for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[db][rb][4 * g4 + e] * inv);
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
          o4.x = oacc[db][rb][4 * g4 + 0];
          o4.y = oacc[db][rb][4 * g4 + 1];
          o4.z = oacc[db][rb][4 * g4 + 2];
          o4.w = oacc[db][rb][4 * g4 + 3];
          *reinterpret_cast<float4 *>(po + 32 * db + 8 * g4 + 4 * hh) = o4;
        }
      if (hh == 0) {
        slot[(size_t)BM * D + lr] = m_run[rb];
        slot[(size_t)BM * D + BM + lr] = l_tot;
      }
    }
  }
}

// --------------------------------------------------------------------------
// Split-KV merge: out = sum_s e^{(m_s-m)c} O_s / sum_s e^{(m_s-m)c} l_s with
// m = max_s m_s (the associative log-sum-exp combine of softmax partials).
// One workgroup of D/4 x ROWS threads merges ROWS rows; a thread owns 4 dims.
// --------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void split_reduce_kernel(
    const float *__restrict__ partials, __bf16 *__restrict__ out,
    const ReduceGroup *__restrict__ groups, int tile_rows, int Hq, int Hkv, float scale_log2e) {
  constexpr int TPR = D / 4;                      // threads per row
  constexpr int ROWS = 256 / TPR;
  const ReduceGroup g = groups[blockIdx.x];
  const int G = Hq / Hkv;
  const int rows_total = g.suffix * G;
  const int lr = blockIdx.y * ROWS + threadIdx.x / TPR;
  const int c4 = (threadIdx.x % TPR) * 4;
  const int row = g.row0 + lr;
  if (lr >= tile_rows || row >= rows_total) return;
  const size_t slot_f = (size_t)tile_rows * (D + 2);
  float m = -INFINITY;
  for (int s = 0; s < g.nsplit; ++s) {
    const float *slot = partials + (size_t)(g.first_slot + s) * slot_f;
    m = fmaxf(m, slot[(size_t)tile_rows * D + lr]);
  }
  float l = 0.f;
  float4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < g.nsplit; ++s) {
    const float *slot = partials + (size_t)(g.first_slot + s) * slot_f;
    const float ms = slot[(size_t)tile_rows * D + lr];
    const float ls = slot[(size_t)tile_rows * D + tile_rows + lr];
    const float w = fast_exp2((ms - m) * scale_log2e);
    const float4 o = *reinterpret_cast<const float4 *>(slot + (size_t)lr * D + c4);
    l += w * ls;
    acc.x += w * o.x;
    acc.y += w * o.y;
    acc.z += w * o.z;
    acc.w += w * o.w;
  }
  const float inv = 1.0f / l;
  const int tok = row / G, gi = row % G;
  __bf16 *op = out + ((int64_t)(g.q_off + tok) * Hq + g.kv_head * G + gi) * D + c4;
  bf16x4 o4;
  o4[0] = (__bf16)(acc.x * inv);
  o4[1] = (__bf16)(acc.y * inv);
  o4[2] = (__bf16)(acc.z * inv);
  o4[3] = (__bf16)(acc.w * inv);
  *reinterpret_cast<bf16x4 *>(op) = o4;
}

template <int D, int RB, int NW, int WPE, int NS>
static int launch_attn_t(const LaunchParams &p, hipStream_t st) {
  constexpr size_t lds_bytes = (size_t)2 * NS * kTileKeys * D * 2;
  auto kernel = prefill_attn_kernel<D, RB, NW, WPE, NS>;
  static const hipError_t attr = hipFuncSetAttribute(
      (const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (attr != hipSuccess) return (int)attr;
  return launch_kernel(kernel, dim3((unsigned)p.num_items), dim3(NW * 64), lds_bytes, st,
                       (const __bf16 *)p.q, (const __bf16 *)p.k_pool, (const __bf16 *)p.v_pool,
                       p.block_table, (__bf16 *)p.out, p.partials, p.items, p.Hq, p.Hkv, p.max_blocks,
                       p.scale_log2e);
}

// Tile shapes: 64 and 128 query rows run two workgroups per CU with two-slot
// rings (64 KB at d=128); 256 rows run one eight-wave workgroup per CU that
// shares every K/V tile among twice as many rows and spends 128 of the 160 KB
// of LDS on four-slot rings.
int launch_attention(const LaunchParams &p, void *stream) {
  if (p.num_items == 0) return 0;
  hipStream_t st = (hipStream_t)stream;
  if (p.rows_per_wave == 64) return launch_attention64(p, stream);
  if (p.d == 128) {
    if (p.tile_rows == 64) return launch_attn_t<128, 1, 2, 2, 2>(p, st);
    if (p.tile_rows == 128) return launch_attn_t<128, 1, 4, 2, 2>(p, st);
    return launch_attn_t<128, 1, 8, 2, 4>(p, st);
  }
  if (p.tile_rows == 64) return launch_attn_t<64, 1, 2, 2, 2>(p, st);
  if (p.tile_rows == 128) return launch_attn_t<64, 1, 4, 2, 2>(p, st);
  return launch_attn_t<64, 1, 8, 2, 4>(p, st);
}

int launch_reduce(const LaunchParams &p, void *stream) {
  if (p.num_groups == 0) return 0;
  hipStream_t st = (hipStream_t)stream;
  if (p.d == 128) {
    dim3 grid((unsigned)p.num_groups, (unsigned)((p.tile_rows + 7) / 8));
    return launch_kernel(split_reduce_kernel<128>, grid, dim3(256), 0, st, (const float *)p.partials,
                         (__bf16 *)p.out, p.groups, p.tile_rows, p.Hq, p.Hkv, p.scale_log2e);
  } else {
    dim3 grid((unsigned)p.num_groups, (unsigned)((p.tile_rows + 15) / 16));
    return launch_kernel(split_reduce_kernel<64>, grid, dim3(256), 0, st, (const float *)p.partials,
                         (__bf16 *)p.out, p.groups, p.tile_rows, p.Hq, p.Hkv, p.scale_log2e);
  }
}

// --------------------------------------------------------------------------
// Machine ceilings as this chip delivers them, for reporting beside the
// published peaks: a register-only MFMA loop and a streaming read.
__global__ __launch_bounds__(256, 2) void mfma_peak_kernel(const bf16x8 *__restrict__ src, float *sink, int iters) {
  // operands come from the caller's buffer: what the matrix pipes sustain
  // depends on the values (constant operands switch far fewer gates than
  // random ones, and the chip's power management sets the clock accordingly)
  const bf16x8 a = src[threadIdx.x], b = src[256 + threadIdx.x];
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[j % 4], 0, 0, 0);
  }
  float r = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int q = 0; q < 16; ++q) r += acc[i][q];
  if (r == -1.0f && iters < 0) sink[0] = r;       // never true: keeps the loop alive
}

__global__ __launch_bounds__(256) void read_peak_kernel(const u32x4 *__restrict__ src, size_t n_vec, float *sink) {
  u32x4 acc = {0u, 0u, 0u, 0u};
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride) {
    const u32x4 v = __builtin_nontemporal_load(src + i);
    acc[0] ^= v[0]; acc[1] ^= v[1]; acc[2] ^= v[2]; acc[3] ^= v[3];
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u && n_vec == 1) sink[0] = 1.f;   // practically never
}

int launch_mfma_peak(const void *src, float *sink, int iters, int *waves, void *stream) {
  const int blocks = 2 * kNumCU;
  *waves = blocks * 4;
  return launch_kernel(mfma_peak_kernel, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const bf16x8 *)src, sink,
                       iters);
}

int launch_read_peak(const void *src, size_t bytes, float *sink, void *stream) {
  return launch_kernel(read_peak_kernel, dim3(16 * kNumCU), dim3(256), 0, (hipStream_t)stream,
                       (const u32x4 *)src, bytes / 16, sink);
}

}  // namespace prism
