// K6: sparse-query causal grouped-query attention on the matrix cores (bf16, head_dim 128).
//
// Queries are the active rows of a layer: arbitrary ascending positions of one sequence.  A workgroup
// takes one tile of 32 query rows and one KV head; wavefront g of the workgroup serves query head
// kv_head * G + g, so all G heads of the group share every K/V tile that is staged in LDS.
//
// Per KV tile of 64 keys a wavefront computes, with 32x32x16 MFMA blocks,
//   S^T[key][q] = K[key][:] . Q[q][:]          (A = K rows from LDS, B = Q held in registers)
//   O^T[d][q]  += V^T[d][key] * P[key][q]      (A = V^T from LDS,    B = P straight from S^T's registers)
// Computing the transposed score tile puts a query's 64 scores into the two lanes (q, q+32), so the
// running softmax needs one cross-lane exchange per tile, and the accumulator layout of S^T is
// already the B-operand layout of the second product up to a fixed permutation of the keys inside
// each group of 16.  V is transposed while it is written to LDS, with that same permutation applied,
// so each operand is one 16-byte LDS read.
//
// LDS rows are padded by 16 bytes (K: 272, V^T: 144 bytes apart) so that operand fetches are free of
// bank conflicts and all LDS addresses are constants off a per-thread base.  K/V rows come from the paged
// cache through the block table, one tile ahead in registers and one tile ahead in a second pair of LDS
// buffers, so a tile costs one barrier.
// KV tiles entirely above the tile's last query position are skipped; the causal mask is applied
// only in tiles that reach above the tile's first query position.  Workgroups are issued longest
// first over the whole launch (KV head fastest, query tiles by decreasing KV range).
#include <type_traits>

#include "common.h"

namespace rc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(float)))) float f32x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

static constexpr int BQ = 32;    // query rows per workgroup
static constexpr int BKV = 64;   // keys per tile
static constexpr int DH = 128;
static constexpr int KROW = DH * 2 + 16;   // bytes between K rows in LDS
static constexpr int VROW = BKV * 2 + 16;  // bytes between V^T rows in LDS
static constexpr int K_TILE_BYTES = BKV * KROW;
static constexpr int V_TILE_BYTES = DH * VROW;
static constexpr int kLdsTableEntries = 2048;   // block-table entries of the workgroup's KV range kept in LDS (paged caches)
static constexpr int ATTN_LDS_BYTES = 2 * (K_TILE_BYTES + V_TILE_BYTES) + kLdsTableEntries * 4;
static constexpr int PROW = DH + 16;         // floats between the rows of a partial result (see attention_partial_floats)
static constexpr int kFragAhead = 4;       // LDS operand fragments in flight ahead of the MFMA that uses them
static constexpr float kRescaleSlack = 8.f;   // log2 units the running maximum may lead the reference exponent

// Maximum over the lane pair (l, l ^ 32).  v_permlane32_swap exchanges the upper half of its first operand with
// the lower half of its second; fed the same value twice it returns (lower half, lower half) and (upper half,
// upper half), so the maximum of the two results is the pair's maximum in every lane, without an LDS round trip.
__device__ inline float pair_max32(float x) {
  const unsigned u = __float_as_uint(x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

// SCORES: additionally write every visible score q.k / sqrt(dh) of every valid row to
// scores[(row * n_q_heads + head) * scores_len + key] (the decode-side influence accumulation reads them), and
// the row's reference exponent and sum, score_ml[row * n_q_heads + head], unless the tile's KV range is split
// (then attn_merge_kernel writes the merged pair).
template <int G, bool SCORES>
__global__ void __launch_bounds__(64 * (G < 4 ? 4 : G), (G <= 4 ? 2 : 1))
attn_mfma_kernel(const bf16* __restrict__ q, const int* __restrict__ row_pos, const ReqTable* __restrict__ table,
                 int fixed_seq, int total_rows, int total_tiles, const bf16* __restrict__ k_pool,
                 const bf16* __restrict__ v_pool, KvGeom g, bf16* __restrict__ out, AttnSplit sp,
                 float* __restrict__ part_o, float2* __restrict__ part_ml, float* __restrict__ scores,
                 int scores_len, float2* __restrict__ score_ml) {
  // A workgroup has at least four wavefronts: with fewer, each thread would stage so much of a K/V tile that the
  // kernel runs out of registers.  In a group of one to three query heads the wavefronts beyond the group only take
  // their share of the staging; they multiply zeros for head 0 of the group and write nothing.
  constexpr int NW = G < 4 ? 4 : G;
  constexpr int NT = 64 * NW;
  // K rows are 256 + 16 bytes, V^T rows 128 + 16 bytes apart.  With 64 banks of 4 bytes, the 16 lanes
  // that fetch the same 16-byte chunk of 16 consecutive rows then hit every bank exactly once, and every
  // LDS address in the main loop is a per-thread base plus a compile-time constant.
  // Two K and two V^T buffers: tile t lives in buffer t % 2 and tile t + 1 is staged while tile t is multiplied,
  // so one barrier per tile suffices.
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_attn[];
  unsigned char* const lds_k = lds_attn;                         // [2][BKV * KROW]
  unsigned char* const lds_vt = lds_attn + 2 * K_TILE_BYTES;     // [2][DH * VROW]

  // late tiles see the most keys: start them first.  With sp.n_chunks > 1 the KV range of a long query
  // tile is cut into chunks of sp.chunk_tiles tiles, one workgroup each, whose partial results are merged
  // by attn_merge_kernel; short tiles are done whole by their chunk-0 workgroup.
  // The KV head varies fastest: workgroups are then dispatched in order of decreasing KV range over the whole
  // grid (a longest-first schedule), and with 8 KV heads every XCD (workgroup id mod 8) keeps to one head's K/V.
  const int kvh = (int)blockIdx.x % g.n_kv_heads;
  const int item = (int)blockIdx.x / g.n_kv_heads;
  const int n_q_heads = g.n_kv_heads * G;
  int r0, n_valid, seq, chunk, split_tile, part_base = 0;   // split_tile < 0: this tile is never split
  if (table) {
    // Work items: requests last to first; inside a request first the query tiles that may be split (one item per
    // tile and KV chunk), then the whole tiles, late ones first.  The host's counts may be upper bounds
    // (rows selected on the device): the table has the live ones.
    if (item >= table->total_items) return;
    int b = table->n_req - 1;                              // item_base is 0 for the last request and grows towards the first
    while (b > 0 && item >= table->r[b - 1].item_base) --b;
    const ReqDev& rq = table->r[b];
    const int tiles = (rq.n_rows + BQ - 1) / BQ;
    const int start = min(rq.long_tile_start, tiles);
    const int j = item - rq.item_base;
    const int n_split_items = (tiles - start) * sp.n_chunks;
    int lt;
    if (j < n_split_items) {
      // chunk-major: chunk 0 of every such tile (late tiles first), then chunk 1, ...  Tiles whose range ends before a
      // chunk have nothing to do there; in this order those empty items sit together at the end of each chunk's run
      // instead of at every n_chunks-th position of the grid (where, for even chunk counts, they kept landing on the
      // same half of the machine and left the other half with all the work)
      chunk = j / (tiles - start);
      lt = tiles - 1 - j % (tiles - start);
    } else {
      lt = start - 1 - (j - n_split_items);
      chunk = 0;
    }
    if (lt < 0) return;
    r0 = rq.row_base + lt * BQ;
    n_valid = min(BQ, rq.row_base + rq.n_rows - r0);
    seq = rq.dst_seq;
    split_tile = lt - rq.long_tile_start;
    part_base = rq.part_base;
  } else {
    chunk = item / total_tiles;
    const int tile = total_tiles - 1 - item % total_tiles;
    if (chunk >= sp.n_chunks) return;
    r0 = tile * BQ;
    n_valid = min(BQ, total_rows - r0);
    seq = fixed_seq;
    split_tile = tile;
  }
  if (n_valid <= 0) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ql = lane & 31, half = lane >> 5;
  const bool active = G >= 4 || wave < G;   // wave-uniform
  const int head = kvh * G + (active ? wave : 0);
  const bool q_ok = active && ql < n_valid;
  const int my_row = r0 + (q_ok ? ql : 0);
  const int my_pos = q_ok ? row_pos[my_row] : 0;
  const int first_pos = row_pos[r0];
  const int last_pos = row_pos[r0 + n_valid - 1];

  // Q as B operands: lane (q, half) holds Q[q][16 s + 8 half .. +7], s = 0..7
  bf16x8 qf[8];
  {
    const bf16* qrow = q + ((size_t)my_row * n_q_heads + head) * DH + 8 * half;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      uint4 v = q_ok ? *reinterpret_cast<const uint4*>(qrow + 16 * s) : make_uint4(0, 0, 0, 0);
      qf[s] = __builtin_bit_cast(bf16x8, v);
    }
  }

  f32x16 acc_o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc_o[i][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c_scale = 1.4426950408889634f / sqrtf((float)DH);   // log2(e) / sqrt(dh)

  // K/V tile staging: every thread owns KPER 16-byte chunks of the K tile (rows krow0 + i*KSTEP, chunk
  // tid%16) and VPER blocks of the V tile (4 consecutive keys x 8 d).  The next tile is fetched into
  // registers while the current one is multiplied.
  constexpr int KSTEP = NT / 16;
  constexpr int KPER = (BKV + KSTEP - 1) / KSTEP;
  constexpr int VPER = (16 + KSTEP - 1) / KSTEP;
  const int krow0 = tid >> 4, kch = tid & 15;      // K: row, 16-byte chunk
  const int vdch0 = tid >> 4, vquad = tid & 15;    // V: chunk of 8 d, quad of 4 keys
  const bool contig = g.max_blocks == 1;           // one block per sequence: rows are a linear function of pos
  const bf16 *kbase = nullptr, *vbase = nullptr;
  if (contig) {
    const size_t o = kv_row_offset(g, seq, 0, kvh);
    kbase = k_pool + o + kch * 8;
    vbase = v_pool + o;
  }
  // Paged cache with power-of-two blocks: the block ids of this workgroup's KV range are copied into LDS once
  // (lds_tab, filled below when the range is known), so that a row's address costs one LDS read instead of a
  // block-table load from memory in front of every K/V load (a dependent pair of global loads has twice the
  // latency the one-tile look-ahead of the fetches has to cover).  Ranges with more blocks than fit, and block
  // sizes that are no power of two, take the general path.
  int* const lds_tab = reinterpret_cast<int*>(lds_attn + 2 * (K_TILE_BYTES + V_TILE_BYTES));
  bool tab_in_lds = false;
  int tab_first = 0;                               // block index of lds_tab[0]
  // lds_tab[i] = block id * n_kv_heads + this workgroup's KV head: the pool row of a position is then a shift and an or
  auto row_offset = [&](int pos) -> size_t {
    if (!tab_in_lds) return kv_row_offset(g, seq, pos, kvh);
    const unsigned e = (unsigned)lds_tab[(pos >> g.bs_shift) - tab_first];
    return ((((size_t)e) << g.bs_shift) | (unsigned)(pos & (g.block_size - 1))) * (size_t)DH;
  };
  // the tile fetched during step t is staged during step t + 1 and multiplied in step t + 2
  uint4 rk[KPER], rv[VPER][4];
  // contiguous cache: this thread's first K chunk and V block of KV tile 0; a full tile is then fetched at constant
  // offsets from one pointer per operand, without per-row position arithmetic or predicates
  const bf16* const kthread = contig ? kbase + (size_t)krow0 * DH : nullptr;
  const bf16* const vthread = contig ? vbase + (size_t)(vquad * 4) * DH + vdch0 * 8 : nullptr;
  // only where every thread owns whole rows / blocks of the tile and registers allow (groups of four query heads; for
  // a group of five the same short-cut gained 4 % on dense layers and lost 3 % on sparse ones)
  constexpr bool kFastFetch = G >= 4 && KPER * KSTEP == BKV && VPER * KSTEP == 16;
  auto fetch_k = [&](int kv0) {
    const bool full = kv0 + BKV - 1 <= last_pos;   // uniform: only a query tile's last KV tile can be ragged
    if (kFastFetch && contig && full) {
      const bf16* kp = kthread + (size_t)kv0 * DH;
#pragma unroll
      for (int i = 0; i < KPER; ++i) rk[i] = *reinterpret_cast<const uint4*>(kp + (size_t)i * KSTEP * DH);
      return;
    }
#pragma unroll
    for (int i = 0; i < KPER; ++i) {
      const int row = krow0 + i * KSTEP;
      const int pos = kv0 + row;
      rk[i] = make_uint4(0, 0, 0, 0);
      if (row < BKV && (full || pos <= last_pos)) {
        const bf16* src = contig ? kbase + (size_t)pos * DH : k_pool + row_offset(pos) + kch * 8;
        rk[i] = *reinterpret_cast<const uint4*>(src);
      }
    }
  };
  auto fetch_v = [&](int kv0) {
    const bool full = kv0 + BKV - 1 <= last_pos;
    if (kFastFetch && contig && full) {
      const bf16* vp = vthread + (size_t)kv0 * DH;
#pragma unroll
      for (int i = 0; i < VPER; ++i)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) rv[i][kk] = *reinterpret_cast<const uint4*>(vp + (size_t)i * KSTEP * 8 + (size_t)kk * DH);
      return;
    }
#pragma unroll
    for (int i = 0; i < VPER; ++i) {
      const int dch = vdch0 + i * KSTEP;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int pos = kv0 + vquad * 4 + kk;
        rv[i][kk] = make_uint4(0, 0, 0, 0);
        if (dch < 16 && (full || pos <= last_pos)) {
          const bf16* src = contig ? vbase + (size_t)pos * DH + dch * 8 : v_pool + row_offset(pos) + dch * 8;
          rv[i][kk] = *reinterpret_cast<const uint4*>(src);
        }
      }
    }
  };
  // V transposed: key = 16 grp + 8 a + 4 h + c goes to column 16 grp + 8 h + 4 a + c; a quad shares (grp, a, h)
  const int vkey0 = vquad * 4;
  const int vcol = (vkey0 & ~15) + 8 * ((vkey0 >> 2) & 1) + 4 * ((vkey0 >> 3) & 1);
  unsigned char* const k_wr = lds_k + krow0 * KROW + kch * 16;
  unsigned char* const v_wr = lds_vt + vdch0 * 8 * VROW + vcol * 2;
  auto stage_k = [&](auto buf) {
    constexpr int KOFF = decltype(buf)::value * K_TILE_BYTES;
#pragma unroll
    for (int i = 0; i < KPER; ++i)
      if (krow0 + i * KSTEP < BKV) *reinterpret_cast<uint4*>(k_wr + KOFF + i * KSTEP * KROW) = rk[i];
  };
  // V^T rows e_begin .. e_end - 1 (of the 8 head-dim elements a thread's block covers)
  auto stage_v = [&](auto buf, int e_begin, int e_end) {
    constexpr int VOFF = decltype(buf)::value * V_TILE_BYTES;
#pragma unroll
    for (int i = 0; i < VPER; ++i) {
      if (vdch0 + i * KSTEP >= 16) continue;
      const uint32_t w[4][4] = {{rv[i][0].x, rv[i][0].y, rv[i][0].z, rv[i][0].w},
                                {rv[i][1].x, rv[i][1].y, rv[i][1].z, rv[i][1].w},
                                {rv[i][2].x, rv[i][2].y, rv[i][2].z, rv[i][2].w},
                                {rv[i][3].x, rv[i][3].y, rv[i][3].z, rv[i][3].w}};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (e < e_begin || e >= e_end) continue;
        const int wi = e >> 1;
        // byte select: even e packs the low halves of two words, odd e the high halves
        const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
        uint2 pk;
        pk.x = __builtin_amdgcn_perm(w[1][wi], w[0][wi], sel);
        pk.y = __builtin_amdgcn_perm(w[3][wi], w[2][wi], sel);
        *reinterpret_cast<uint2*>(v_wr + VOFF + (i * KSTEP * 8 + e) * VROW) = pk;
      }
    }
  };
  // operand fetch addresses: K block b, dh step s -> k_rd + b*32*KROW + s*32 ; V^T block db, key step tt
  const unsigned char* const k_rd = lds_k + ql * KROW + half * 16;
  const unsigned char* const v_rd = lds_vt + ql * VROW + half * 16;

  const int n_kv_tiles = last_pos / BKV + 1;
  const bool is_split = sp.n_chunks > 1 && split_tile >= 0 && n_kv_tiles > sp.long_thr;
  const int t_begin = is_split ? chunk * sp.chunk_tiles : 0;
  const int t_end = is_split ? min(n_kv_tiles, t_begin + sp.chunk_tiles) : n_kv_tiles;
  if (t_begin >= t_end || (!is_split && chunk != 0)) return;   // nothing for this workgroup (uniform)
  if (!contig && g.bs_shift >= 0) {
    tab_first = (t_begin * BKV) >> g.bs_shift;
    const int n_blk = min(((t_end * BKV - 1) >> g.bs_shift), g.max_blocks - 1) - tab_first + 1;
    if (n_blk <= kLdsTableEntries) {   // uniform
      for (int i = tid; i < n_blk; i += NT) {
        const int blk = g.block_table[(size_t)seq * g.max_blocks + tab_first + i];
        lds_tab[i] = min(max(blk, 0), g.n_blocks - 1) * g.n_kv_heads + kvh;
      }
      tab_in_lds = true;
      __syncthreads();
    }
  }
  const std::integral_constant<int, 0> buf0;
  const std::integral_constant<int, 1> buf1;
  // prologue: the first tile goes to buffer 0, the second one is on its way in registers
  fetch_k(t_begin * BKV);
  fetch_v(t_begin * BKV);
  stage_k(buf0);
  stage_v(buf0, 0, 8);
  if (t_begin + 1 < t_end) {
    fetch_k((t_begin + 1) * BKV);
    fetch_v((t_begin + 1) * BKV);
  }
  __syncthreads();
  // step i (tile t = t_begin + i) multiplies buffer i % 2; meanwhile it stages tile t + 1 into the other buffer
  // (free since the barrier that ended step i - 1) and starts the loads of tile t + 2.  That staging is vector-ALU
  // and LDS-write work, which is dealt out between the MFMAs of S^T so that it runs while the matrix pipe is busy.
  auto tile_step = [&](int t, auto buf) {
    constexpr int KOFF = decltype(buf)::value * K_TILE_BYTES, VOFF = decltype(buf)::value * V_TILE_BYTES;
    const std::integral_constant<int, 1 - decltype(buf)::value> other;
    const int kv0 = t * BKV;
    const bool has_next = t + 1 < t_end, has_next2 = t + 2 < t_end;
    auto staging_slice = [&](int i) {   // i-th of the 16 gaps between the MFMAs of S^T
      if (!has_next) return;
      if (i == 0) stage_k(other);
      else if (i >= 1 && i <= 4) stage_v(other, 2 * (i - 1), 2 * i);
    };

    // S^T = K Q^T : two blocks of 32 keys.  The two accumulator chains alternate and the K fragments are read
    // kFragAhead MFMAs ahead of their use, so that neither the LDS latency nor the MFMA dependency is exposed.
    f32x16 acc_s[2];
    {
      f32x16 zero;   // the first product of each chain takes a constant-zero accumulator: no registers to clear
#pragma unroll
      for (int e = 0; e < 16; ++e) zero[e] = 0.f;
      auto k_frag = [&](int i) {   // step i: key block i & 1, head-dim step i >> 1
        return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(k_rd + KOFF + (i & 1) * 32 * KROW + (i >> 1) * 32));
      };
      bf16x8 kf[kFragAhead];
#pragma unroll
      for (int i = 0; i < kFragAhead; ++i) kf[i] = k_frag(i);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        acc_s[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i % kFragAhead], qf[i >> 1], i < 2 ? zero : acc_s[i & 1], 0, 0, 0);
        if (i + kFragAhead < 16) kf[i % kFragAhead] = k_frag(i + kFragAhead);
        staging_slice(i);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (has_next2) {
      fetch_k(kv0 + 2 * BKV);
      fetch_v(kv0 + 2 * BKV);
    }
    // the first V^T fragments do not depend on the softmax: their LDS reads run under it
    auto v_frag = [&](int i) {     // step i: head-dim block i & 3, key step i >> 2
      return __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(v_rd + VOFF + (i & 3) * 32 * VROW + (i >> 2) * 32));
    };
    bf16x8 vf[kFragAhead];
#pragma unroll
    for (int i = 0; i < kFragAhead; ++i) vf[i] = v_frag(i);
    // running softmax on raw scores; the 1/sqrt(dh) * log2(e) factor is folded into the exponent.
    // Element e of block b is key kv0 + 32 b + 8 (e/4) + 4 half + e%4.  Only tiles that reach above the
    // tile's first query position need the causal mask.
    if (kv0 + BKV - 1 > first_pos) {
      asm volatile("; causal mask tile" ::: "memory");   // keeps this a real (wave-uniform) branch
#pragma unroll
      for (int b = 0; b < 2; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int key = kv0 + 32 * b + 8 * (e >> 2) + 4 * half + (e & 3);
          if (key > my_pos) acc_s[b][e] = -INFINITY;
        }
    }
    if (SCORES) {
      if (q_ok) {
        float* srow = scores + ((size_t)my_row * n_q_heads + head) * scores_len;
        const float inv_sqrt = 1.0f / sqrtf((float)DH);
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int key = kv0 + 32 * b + 8 * (e >> 2) + 4 * half + (e & 3);
            if (key <= my_pos) srow[key] = acc_s[b][e] * inv_sqrt;
          }
      }
    }
    float mx = acc_s[0][0];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, acc_s[b][e]);
    mx = pair_max32(mx);
    // m_run is the reference exponent of the running sums, in the scaled (log2) domain.  It follows the
    // running maximum lazily: the sums are rescaled (64 multiplies per lane) only when some row's maximum has
    // grown by more than kRescaleSlack since its last rescale, so p stays below 2^kRescaleSlack instead of 1.
    // Any reference gives the same quotient O / l; bf16 keeps p's relative precision at every magnitude.
    // A row that has not seen a visible key yet keeps m_run = -inf; m_use avoids inf - inf in that case
    // (all its p are then 0).
    const float m_new = fmaxf(m_run, mx * c_scale);
    if (__any(m_new > m_run + kRescaleSlack)) {   // wave-uniform
      const float m_to = (m_new == -INFINITY) ? 0.f : m_new;
      const float corr = __builtin_amdgcn_exp2f(m_run - m_to);
      l_run *= corr;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc_o[i][e] *= corr;
      m_run = m_new;
    }
    const float m_use = (m_run == -INFINITY) ? 0.f : m_run;
    float psum = 0.f;
    bf16x8 pf[4];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        f32x8 p;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          p[j] = __builtin_amdgcn_exp2f(fmaf(acc_s[b][8 * u + j], c_scale, -m_use));
          psum += p[j];
        }
        pf[2 * b + u] = __builtin_convertvector(p, bf16x8);
      }
    l_run += psum;
    // O^T += V^T P : four accumulator chains alternate, fragments read kFragAhead MFMAs ahead
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      acc_o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i % kFragAhead], pf[i >> 2], acc_o[i & 3], 0, 0, 0);
      if (i + kFragAhead < 16) vf[i % kFragAhead] = v_frag(i + kFragAhead);
    }
    __syncthreads();   // tile t fully consumed, tile t + 1 fully staged
  };
  for (int t = t_begin; t < t_end; t += 2) {
    tile_step(t, buf0);
    if (t + 1 < t_end) tile_step(t + 1, buf1);
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (!active) return;
  if (is_split) {
    // partial result of this chunk: un-normalised O, running maximum (log2 domain) and sum
    const size_t slot = ((size_t)(part_base + split_tile * sp.n_chunks + chunk) * n_q_heads + head) * BQ + ql;
    if (half == 0) part_ml[slot] = make_float2(m_run, l_tot);
    float* po = part_o + slot * PROW;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int d = 32 * db + 8 * e4 + 4 * half;
        *reinterpret_cast<float4*>(po + d) = make_float4(acc_o[db][4 * e4 + 0], acc_o[db][4 * e4 + 1],
                                                          acc_o[db][4 * e4 + 2], acc_o[db][4 * e4 + 3]);
      }
    return;
  }
  if (q_ok) {
    if (SCORES && half == 0) score_ml[(size_t)my_row * n_q_heads + head] = make_float2(m_run, l_tot);
    const float inv = 1.0f / l_tot;
    bf16* orow = out + ((size_t)my_row * n_q_heads + head) * DH;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int d = 32 * db + 8 * e4 + 4 * half;
        uint2 pk;
        pk.x = (uint32_t)f32_to_bf16(acc_o[db][4 * e4 + 0] * inv).v | ((uint32_t)f32_to_bf16(acc_o[db][4 * e4 + 1] * inv).v << 16);
        pk.y = (uint32_t)f32_to_bf16(acc_o[db][4 * e4 + 2] * inv).v | ((uint32_t)f32_to_bf16(acc_o[db][4 * e4 + 3] * inv).v << 16);
        *reinterpret_cast<uint2*>(orow + d) = pk;
      }
  }
}

// Merge of the KV chunks of one (row, head): one wavefront each, two head-dim elements per lane.
// Only rows of split tiles take part; chunk c holds keys for a row iff its first key position is <=
// the row's position.
__global__ void __launch_bounds__(256)
attn_merge_kernel(const int* __restrict__ row_pos, const int* __restrict__ row_req, const ReqTable* __restrict__ table,
                  int total_rows, int n_q_heads, AttnSplit sp, const float* __restrict__ part_o,
                  const float2* __restrict__ part_ml, bf16* __restrict__ out, float2* __restrict__ score_ml) {
  const int item = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  int r, head, split_tile, ql, part_base = 0, tile_last_row;
  if (table) {
    // items run over the rows of the tiles that may be split only (the late tiles of every request)
    const int mr = item / n_q_heads;
    head = item - mr * n_q_heads;
    if (mr >= table->total_merge_rows) return;
    int b = 0;
    while (b + 1 < table->n_req && mr >= table->r[b + 1].merge_base) ++b;
    const ReqDev& rq = table->r[b];
    const int local = min(rq.long_tile_start, 1 << 20) * BQ + (mr - rq.merge_base);     // row inside the request
    if (local >= rq.n_rows) return;
    r = rq.row_base + local;
    const int lt = local / BQ;
    split_tile = lt - rq.long_tile_start;
    ql = local % BQ;
    part_base = rq.part_base;
    tile_last_row = min(rq.row_base + (lt + 1) * BQ, rq.row_base + rq.n_rows) - 1;
  } else {
    if (item >= total_rows * n_q_heads) return;
    r = item / n_q_heads;
    head = item - r * n_q_heads;
    split_tile = r / BQ;
    ql = r % BQ;
    tile_last_row = min((split_tile + 1) * BQ, total_rows) - 1;
  }
  const int n_kv_tiles = row_pos[tile_last_row] / BKV + 1;
  if (split_tile < 0 || n_kv_tiles <= sp.long_thr) return;   // this row's tile was done by one workgroup
  const int nc = min(sp.n_chunks, row_pos[r] / (sp.chunk_tiles * BKV) + 1);
  const size_t slot0 = ((size_t)(part_base + split_tile * sp.n_chunks) * n_q_heads + head) * BQ + ql;
  const size_t cstride = (size_t)n_q_heads * BQ;
  // Pass 1, one chunk per lane (64 at a time): the common reference exponent.  Pass 2: every lane needs every
  // chunk's weight, so the (m, l) pairs are read again (they are cached) and the partial outputs of four chunks are
  // requested before the first is used.  The sums run in chunk order.
  float m = -INFINITY;
  for (int c = lane; c < nc; c += 64) m = fmaxf(m, part_ml[slot0 + c * cstride].x);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 64));
  float l = 0.f, o0 = 0.f, o1 = 0.f;
  int c = 0;
  for (; c + 4 <= nc; c += 4) {
    float2 ml[4], o[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const size_t slot = slot0 + (c + u) * cstride;
      ml[u] = part_ml[slot];
      o[u] = *reinterpret_cast<const float2*>(part_o + slot * PROW + 2 * lane);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float wgt = (ml[u].x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ml[u].x - m);
      l += ml[u].y * wgt;
      o0 += o[u].x * wgt;
      o1 += o[u].y * wgt;
    }
  }
  for (; c < nc; ++c) {
    const size_t slot = slot0 + c * cstride;
    const float2 ml = part_ml[slot];
    const float wgt = (ml.x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ml.x - m);
    l += ml.y * wgt;
    const float2 o = *reinterpret_cast<const float2*>(part_o + slot * PROW + 2 * lane);
    o0 += o.x * wgt;
    o1 += o.y * wgt;
  }
  if (score_ml && lane == 0) score_ml[(size_t)r * n_q_heads + head] = make_float2(m, l);
  const float inv = 1.0f / l;
  const uint32_t pk = (uint32_t)f32_to_bf16(o0 * inv).v | ((uint32_t)f32_to_bf16(o1 * inv).v << 16);
  *reinterpret_cast<uint32_t*>(out + ((size_t)r * n_q_heads + head) * DH + 2 * lane) = pk;
}

static int g_force_chunk_tiles = 0;   // 0: by shape; > 0: this many KV tiles per chunk
void set_attention_chunk_tiles(int t) { g_force_chunk_tiles = t; }
int attention_forced_chunk_tiles() { return g_force_chunk_tiles; }

// Partial results: per (slot, head, query row) DH un-normalised output floats, stored PROW floats apart, and one
// (reference exponent, sum) pair behind all of them.  The row pitch is not a power of two on purpose: with 512-byte
// rows the slots of one KV chunk of successive query tiles lie a multiple of 1 MiB apart whenever the chunk count is
// even, and the workgroups that finish together (same chunk, neighbouring tiles) then write to the same memory
// channels (measured: even chunk counts ran the split layers up to twice as slow).
size_t attention_partial_floats(int total_slots, int n_q_heads) {
  return (size_t)total_slots * n_q_heads * BQ * (PROW + 2);
}

template <int G>
static hipError_t launch_g(const bf16* q, const int* row_pos, const ReqTable* table, int fixed_seq, int total_rows,
                           int total_tiles, const bf16* k_pool, const bf16* v_pool, KvGeom g, bf16* out,
                           AttnSplit sp, float* part, float* scores, int scores_len, hipStream_t st) {
  // with a table, total_tiles is the phase's number of work items (ReqTable::total_items, or an upper bound of it)
  const long items = table ? (long)total_tiles : (long)total_tiles * sp.n_chunks;
  dim3 grid((unsigned)(items * g.n_kv_heads));
  float* part_o = part;
  float2* part_ml = reinterpret_cast<float2*>(part + (size_t)sp.total_slots * g.n_kv_heads * G * BQ * PROW);
  // more than the 64 KB a kernel gets without asking
  static std::atomic<unsigned long long> told_scores{0}, told_plain{0};
  hipError_t e = scores ? allow_dynamic_lds((const void*)attn_mfma_kernel<G, true>, ATTN_LDS_BYTES, told_scores)
                        : allow_dynamic_lds((const void*)attn_mfma_kernel<G, false>, ATTN_LDS_BYTES, told_plain);
  if (e != hipSuccess) return e;
  if (scores)
    attn_mfma_kernel<G, true><<<grid, 64 * (G < 4 ? 4 : G), ATTN_LDS_BYTES, st>>>(q, row_pos, table, fixed_seq, total_rows, total_tiles, k_pool,
                                                                    v_pool, g, out, sp, part_o, part_ml, scores, scores_len,
                                                                    influence_pairs(scores, total_rows, g.n_kv_heads * G, scores_len));
  else
    attn_mfma_kernel<G, false><<<grid, 64 * (G < 4 ? 4 : G), ATTN_LDS_BYTES, st>>>(q, row_pos, table, fixed_seq, total_rows, total_tiles, k_pool,
                                                                     v_pool, g, out, sp, part_o, part_ml, nullptr, 0, nullptr);
  return hipGetLastError();
}

hipError_t launch_attention_bf16(const bf16* q, const int* row_pos, const int* row_req, const ReqTable* table,
                                 int fixed_seq, int total_rows, int total_tiles, const bf16* k_pool,
                                 const bf16* v_pool, KvGeom g, int n_q_heads, bf16* out, AttnSplit sp, float* part,
                                 hipStream_t st, float* scores, int scores_len, int merge_rows) {
  if (total_rows <= 0) return hipSuccess;
  const int G = n_q_heads / g.n_kv_heads;
  if (!part || sp.total_slots <= 0) sp = attention_no_split();
  hipError_t e;
  switch (G) {
#define RC_ATTN_CASE(GG) \
    case GG: e = launch_g<GG>(q, row_pos, table, fixed_seq, total_rows, total_tiles, k_pool, v_pool, g, out, sp, part, scores, scores_len, st); break;
    RC_ATTN_CASE(1) RC_ATTN_CASE(2) RC_ATTN_CASE(3) RC_ATTN_CASE(4)
    RC_ATTN_CASE(5) RC_ATTN_CASE(6) RC_ATTN_CASE(7) RC_ATTN_CASE(8)
#undef RC_ATTN_CASE
    default:  // wider groups: one wavefront per (row, head) on the vector ALUs
      if (scores) return hipErrorInvalidValue;
      return launch_attention_simt<bf16>(q, row_pos, row_req, table, fixed_seq, total_rows, k_pool, v_pool, g,
                                         n_q_heads, out, st);
  }
  if (e != hipSuccess || sp.n_chunks == 1) return e;
  const float2* part_ml = reinterpret_cast<const float2*>(part + (size_t)sp.total_slots * n_q_heads * BQ * PROW);
  // with a table, merge_rows (the rows of the tiles that may be split, or an upper bound) sizes the merge grid
  const int items = (table ? merge_rows : total_rows) * n_q_heads;
  if (items <= 0) return hipSuccess;
  attn_merge_kernel<<<(items + 3) / 4, 256, 0, st>>>(row_pos, row_req, table, total_rows, n_q_heads, sp, part, part_ml,
                                                     out, scores ? influence_pairs(scores, total_rows, n_q_heads, scores_len) : nullptr);
  return hipGetLastError();
}

template <>
hipError_t launch_attention<bf16>(const bf16* q, const int* row_pos, const int* row_req, const ReqTable* table,
                                  int fixed_seq, int total_rows, int total_tiles, const bf16* k_pool,
                                  const bf16* v_pool, KvGeom g, int n_q_heads, bf16* out, hipStream_t st) {
  const AttnSplit sp = attention_no_split();
  return launch_attention_bf16(q, row_pos, row_req, table, fixed_seq, total_rows, total_tiles, k_pool, v_pool, g,
                               n_q_heads, out, sp, nullptr, st);
}

}  // namespace rc
