// HIP kernels for gfx950 (CDNA4): paged KV append, paged flash-style prefill
// attention with bf16 MFMA, and the split-KV merge.
//
// What is computed follows the paper's statement of prefix reuse (Sec. 2.2,
// Eq. 3-4): the uncached suffix rows of each request attend causally over the
// cached prefix KV (gathered through the block table) and over their own KV.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "prism_internal.h"

namespace prism {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// --------------------------------------------------------------------------
// Paged KV append.  One thread moves 16 bytes of K and 16 bytes of V.
// --------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void kv_append_kernel(
    const u32x4 *__restrict__ k_src, const u32x4 *__restrict__ v_src, u32x4 *__restrict__ k_pool,
    u32x4 *__restrict__ v_pool, const int32_t *__restrict__ block_table,
    const TokInfo *__restrict__ toks, int num_tokens, int Hkv, int max_blocks) {
  constexpr int CH = D / 8;                       // 16-byte chunks per (token, head) row
  const int64_t per_tok = (int64_t)Hkv * CH;
  const int64_t total = (int64_t)num_tokens * per_tok;
  for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < total;
       c += (int64_t)gridDim.x * blockDim.x) {
    const int tok = (int)(c / per_tok);
    const int rem = (int)(c - (int64_t)tok * per_tok);
    const int h = rem / CH, ch = rem % CH;
    const TokInfo ti = toks[tok];
    const int32_t page = block_table[(int64_t)ti.req * max_blocks + ti.pos / kPage];
    const int64_t dst = (((int64_t)page * Hkv + h) * kPage + (ti.pos % kPage)) * CH + ch;
    k_pool[dst] = k_src[c];
    v_pool[dst] = v_src[c];
  }
}

int launch_append(const void *k_src, const void *v_src, void *k_pool, void *v_pool,
                  const int32_t *block_table, const TokInfo *toks, int num_tokens, int Hkv, int d,
                  int max_blocks, void *stream) {
  if (num_tokens == 0) return 0;
  const int64_t total = (int64_t)num_tokens * Hkv * (d / 8);
  int64_t blocks = (total + 255) / 256;
  if (blocks > 16 * 1024) blocks = 16 * 1024;
  dim3 grid((unsigned)blocks), block(256);
  hipStream_t st = (hipStream_t)stream;
  if (d == 128)
    hipLaunchKernelGGL(kv_append_kernel<128>, grid, block, 0, st, (const u32x4 *)k_src,
                       (const u32x4 *)v_src, (u32x4 *)k_pool, (u32x4 *)v_pool, block_table, toks,
                       num_tokens, Hkv, max_blocks);
  else
    hipLaunchKernelGGL(kv_append_kernel<64>, grid, block, 0, st, (const u32x4 *)k_src,
                       (const u32x4 *)v_src, (u32x4 *)k_pool, (u32x4 *)v_pool, block_table, toks,
                       num_tokens, Hkv, max_blocks);
  return (int)hipGetLastError();
}

// --------------------------------------------------------------------------
// Prefill attention.
//
// A workgroup of NW waves owns NW*32*RB packed query rows of one (request, kv
// head) and walks the key range in tiles of 64 keys (four 16-token pages).
// Each tile's K and V rows are copied from the paged pool straight into LDS
// (global_load_lds, 16 bytes per lane, no staging registers) into one of two
// buffers, so the copy of tile t+1 overlaps the math of tile t and there is
// one workgroup barrier per tile.
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

template <int D>
__device__ __forceinline__ int swz(int key) {
  if (D == 128) return ((key & 3) << 2) | ((key >> 2) & 3);
  return (((key >> 1) & 1) << 2) | ((key >> 2) & 3);
}

template <int D>
__device__ __forceinline__ int lds_off(int key, int chunk) {   // byte offset of a 16-byte chunk
  return key * (D * 2) + ((chunk ^ swz<D>(key)) << 4);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr float kRescaleThreshold = 8.0f;   // log2 units

template <int D, int RB, int NW, int WPE>
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

  __shared__ __attribute__((aligned(1024))) unsigned char lds[2][2][TILE_BYTES];   // [buffer][K,V]

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
  // Wave-uniform key bounds: below lo_limit no row of the wave is masked,
  // above hi_limit every row is.
  const int first_row = wrow0 < rows_total ? wrow0 : rows_total - 1;
  int last_row = wrow0 + 32 * RB - 1;
  if (last_row > rows_total - 1) last_row = rows_total - 1;
  const bool wave_live = wrow0 < rows_total;
  const int lo_limit = P + first_row / G;
  const int hi_limit = P + last_row / G;

  f32x16 oacc[DB][RB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[db][rb][r] = 0.f;
  float m_run[RB], l_run[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    m_run[rb] = -1e30f;
    l_run[rb] = 0.f;
  }

  // ---- paged copy: wave w moves units w*UPW .. w*UPW+UPW-1 of the tile; a
  // unit is 1 KB = KPU whole key rows, and consecutive units stay inside one
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
  const int wave_blk = (wave * UPW) / UPP;        // first page of the tile this wave copies from
  auto page_of = [&](int key0, int j) -> int32_t {
    int blk = key0 / kPage + wave_blk + j;
    if (blk > nblk - 1) blk = nblk - 1;           // never read a table entry past the sequence
    return bt[blk];
  };
  auto copy_tile = [&](int buf, const int32_t (&pages)[PPW]) {
#pragma unroll
    for (int i = 0; i < UPW; ++i) {
      const int u = wave * UPW + i;
      const int64_t base = (int64_t)pages[i / UPP] * page_stride + head_off;   // wave-uniform
      const unsigned char *ksrc = (const unsigned char *)k_pool + base;
      const unsigned char *vsrc = (const unsigned char *)v_pool + base;
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void *)(ksrc + lane_src[i]),
          (__attribute__((address_space(3))) void *)(&lds[buf][0][u * 1024]), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void *)(vsrc + lane_src[i]),
          (__attribute__((address_space(3))) void *)(&lds[buf][1][u * 1024]), 16, 0, 0);
    }
  };

  const int kv_begin = it.kv_begin, kv_end = it.kv_end;
  int32_t pages[PPW];
  if (kv_begin < kv_end) {
#pragma unroll
    for (int j = 0; j < PPW; ++j) pages[j] = page_of(kv_begin, j);
    copy_tile(0, pages);
#pragma unroll
    for (int j = 0; j < PPW; ++j) pages[j] = page_of(kv_begin + BN, j);
  }

  int buf = 0;
  for (int key0 = kv_begin; key0 < kv_end; key0 += BN, buf ^= 1) {
    __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's part of the tile has landed
    __syncthreads();                              // everyone's has; the other buffer is free again
    if (key0 + BN < kv_end) {
      copy_tile(buf ^ 1, pages);
#pragma unroll
      for (int j = 0; j < PPW; ++j) pages[j] = page_of(key0 + 2 * BN, j);
    }
    unsigned char *k_lds = &lds[buf][0][0];
    unsigned char *v_lds = &lds[buf][1][0];
    if (key0 + BN > T) {
      // Slots past the end of the sequence hold whatever the pool held: clear
      // those V rows so that 0 * garbage cannot poison the products.
      for (int c = tid; c < BN * CPR; c += NT)
        if (key0 + c / CPR >= T) *reinterpret_cast<u32x4 *>(v_lds + c * 16) = u32x4{0u, 0u, 0u, 0u};
      __syncthreads();
    }

    if (!wave_live || key0 > hi_limit) continue;  // nothing visible to this wave in the tile

    // ---- S^T = K Q^T
    f32x16 sacc[BN / 32][RB];
#pragma unroll
    for (int kb = 0; kb < BN / 32; ++kb)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[kb][rb][r] = 0.f;
#pragma unroll
    for (int kb = 0; kb < BN / 32; ++kb) {
      const int key = kb * 32 + l32;
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(k_lds + lds_off<D>(key, 2 * kk + hh));
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          sacc[kb][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[rb][kk], sacc[kb][rb], 0, 0, 0);
      }
    }

    // ---- causal mask (only tiles that reach past the wave's first row)
    if (key0 + BN - 1 > lo_limit) {
#pragma unroll
      for (int kb = 0; kb < BN / 32; ++kb)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = key0 + kb * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
            if (key > limit[rb]) sacc[kb][rb][r] = -INFINITY;
          }
    }

    // ---- online softmax
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      float mx = sacc[0][rb][0];
#pragma unroll
      for (int kb = 0; kb < BN / 32; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[kb][rb][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const bool grow = (mx - m_run[rb]) * scale_log2e > kRescaleThreshold;
      if (__builtin_amdgcn_ballot_w64(grow) != 0) {
        const float m_new = fmaxf(m_run[rb], mx);
        const float alpha = fast_exp2((m_run[rb] - m_new) * scale_log2e);
        m_run[rb] = m_new;
        l_run[rb] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) oacc[db][rb][r] *= alpha;
      }
      const float mc = m_run[rb] * scale_log2e;
      float sum = 0.f;
#pragma unroll
      for (int kb = 0; kb < BN / 32; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float pv = fast_exp2(fmaf(sacc[kb][rb][r], scale_log2e, -mc));
          sacc[kb][rb][r] = pv;
          sum += pv;
        }
      l_run[rb] += sum;
    }

    // ---- O^T += V^T P^T
#pragma unroll
    for (int ks = 0; ks < BN / 16; ++ks) {
      bf16x8 pf[RB];
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int e = 0; e < 8; ++e) pf[rb][e] = (__bf16)sacc[ks >> 1][rb][8 * (ks & 1) + e];
      // Transposing read: within 16 lanes, lane i supplies the address of 4
      // head dims 4*(i%4).. of key (i/4); it receives 4 keys of head dim i.
      const int i16 = lane & 15;
      const int grp = (lane >> 4) & 1;
      const int keyA = 16 * ks + 4 * hh + (i16 >> 2);
      const int keyB = keyA + 8;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const int chunk = 4 * db + 2 * grp + ((i16 & 3) >> 1);
        const int sub = (i16 & 1) << 3;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4 *)(v_lds + lds_off<D>(keyA, chunk) + sub));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4 *)(v_lds + lds_off<D>(keyB, chunk) + sub));
        union {
          s16x4 h[2];
          bf16x8 v;
        } a;
        a.h[0] = lo;
        a.h[1] = hi;
#pragma unroll
        for (int rb = 0; rb < RB; ++rb)
          oacc[db][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, pf[rb], oacc[db][rb], 0, 0, 0);
      }
    }
  }

  // ---- epilogue
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const int row = wrow0 + rb * 32 + l32;
    const float l_tot = l_run[rb] + __shfl_xor(l_run[rb], 32);
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

template <int D, int RB, int NW, int WPE>
static int launch_attn_t(const LaunchParams &p, hipStream_t st) {
  hipLaunchKernelGGL((prefill_attn_kernel<D, RB, NW, WPE>), dim3((unsigned)p.num_items), dim3(NW * 64), 0,
                     st, (const __bf16 *)p.q, (const __bf16 *)p.k_pool, (const __bf16 *)p.v_pool,
                     p.block_table, (__bf16 *)p.out, p.partials, p.items, p.Hq, p.Hkv, p.max_blocks,
                     p.scale_log2e);
  return (int)hipGetLastError();
}

int launch_attention(const LaunchParams &p, void *stream) {
  if (p.num_items == 0) return 0;
  hipStream_t st = (hipStream_t)stream;
  if (p.d == 128) {
    if (p.tile_rows == 64) return launch_attn_t<128, 1, 2, 2>(p, st);
    if (p.tile_rows == 128) return launch_attn_t<128, 1, 4, 2>(p, st);
    return launch_attn_t<128, 2, 4, 1>(p, st);
  }
  if (p.tile_rows == 64) return launch_attn_t<64, 1, 2, 2>(p, st);
  if (p.tile_rows == 128) return launch_attn_t<64, 1, 4, 2>(p, st);
  return launch_attn_t<64, 2, 4, 1>(p, st);
}

int launch_reduce(const LaunchParams &p, void *stream) {
  if (p.num_groups == 0) return 0;
  hipStream_t st = (hipStream_t)stream;
  if (p.d == 128) {
    dim3 grid((unsigned)p.num_groups, (unsigned)((p.tile_rows + 7) / 8));
    hipLaunchKernelGGL(split_reduce_kernel<128>, grid, dim3(256), 0, st, p.partials, (__bf16 *)p.out,
                       p.groups, p.tile_rows, p.Hq, p.Hkv, p.scale_log2e);
  } else {
    dim3 grid((unsigned)p.num_groups, (unsigned)((p.tile_rows + 15) / 16));
    hipLaunchKernelGGL(split_reduce_kernel<64>, grid, dim3(256), 0, st, p.partials, (__bf16 *)p.out,
                       p.groups, p.tile_rows, p.Hq, p.Hkv, p.scale_log2e);
  }
  return (int)hipGetLastError();
}

}  // namespace prism
