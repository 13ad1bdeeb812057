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
// LDS rows are 8 (K: 16) chunks of 16 bytes; chunk c of row r sits at slot c ^ (r & 7): conflict-free
// for the row-strided operand reads.  K/V rows come from the paged cache through the block table.
// KV tiles entirely above the tile's last query position are skipped; the causal mask is applied
// only in tiles that reach above the tile's first query position.  Workgroups are issued longest
// first.
#include "common.h"

namespace rc {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(float)))) float f32x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

static constexpr int BQ = 32;    // query rows per workgroup
static constexpr int BKV = 64;   // keys per tile
static constexpr int DH = 128;

template <int G>
__global__ void __launch_bounds__(64 * G)
attn_mfma_kernel(const bf16* __restrict__ q, const int* __restrict__ row_pos, const ReqTable* __restrict__ table,
                 int fixed_seq, int total_rows, int total_tiles, const bf16* __restrict__ k_pool,
                 const bf16* __restrict__ v_pool, KvGeom g, bf16* __restrict__ out) {
  constexpr int NT = 64 * G;
  __shared__ uint4 lds_k[BKV * 16];        // [64 keys][16 chunks]
  __shared__ uint4 lds_vt[DH * 8];         // [128 d][8 chunks of 8 (permuted) keys]

  const int tile = total_tiles - 1 - (int)blockIdx.x;   // late tiles see the most keys: start them first
  const int kvh = blockIdx.y;
  const int n_q_heads = g.n_kv_heads * G;
  int r0, n_valid, seq;
  if (table) {
    int b = 0;
    while (b + 1 < table->n_req && tile >= table->r[b + 1].tile_base) ++b;
    const ReqDev& rq = table->r[b];
    r0 = rq.row_base + (tile - rq.tile_base) * BQ;
    n_valid = min(BQ, rq.row_base + rq.n_rows - r0);
    seq = rq.dst_seq;
  } else {
    r0 = tile * BQ;
    n_valid = min(BQ, total_rows - r0);
    seq = fixed_seq;
  }
  if (n_valid <= 0) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ql = lane & 31, half = lane >> 5;
  const int head = kvh * G + wave;
  const bool q_ok = ql < n_valid;
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

  const int n_tiles = last_pos / BKV + 1;
  for (int t = 0; t < n_tiles; ++t) {
    const int kv0 = t * BKV;
    __syncthreads();   // previous tile fully consumed
    // K tile: 64 rows x 16 chunks
    for (int idx = tid; idx < BKV * 16; idx += NT) {
      const int row = idx >> 4, ch = idx & 15;
      const int pos = kv0 + row;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (pos <= last_pos) v = *reinterpret_cast<const uint4*>(k_pool + kv_row_offset(g, seq, pos, kvh) + ch * 8);
      lds_k[row * 16 + (ch ^ (row & 7))] = v;
    }
    // V tile, transposed: item = (quad of 4 consecutive keys, chunk of 8 d)
    for (int idx = tid; idx < (BKV / 4) * 16; idx += NT) {
      const int dch = idx >> 4, quad = idx & 15;   // 16 lanes = 16 quads = 16 distinct 8-byte LDS slots
      uint32_t w[4][4];
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        const int pos = kv0 + quad * 4 + kk;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (pos <= last_pos) v = *reinterpret_cast<const uint4*>(v_pool + kv_row_offset(g, seq, pos, kvh) + dch * 8);
        w[kk][0] = v.x; w[kk][1] = v.y; w[kk][2] = v.z; w[kk][3] = v.w;
      }
      // key = 16 grp + 8 a + 4 h + c  ->  column 16 grp + 8 h + 4 a + c ; a quad shares (grp, a, h)
      const int key0 = quad * 4;
      const int col = (key0 & ~15) + 8 * ((key0 >> 2) & 1) + 4 * ((key0 >> 3) & 1);
      const int chunk = col >> 3, within = (col & 7) >> 2;   // 8-byte half of the 16-byte chunk
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int d = dch * 8 + e;
        const int wi = e >> 1;
        uint2 pk;
        if (e & 1) {
          pk.x = (w[0][wi] >> 16) | (w[1][wi] & 0xffff0000u);
          pk.y = (w[2][wi] >> 16) | (w[3][wi] & 0xffff0000u);
        } else {
          pk.x = (w[0][wi] & 0xffffu) | (w[1][wi] << 16);
          pk.y = (w[2][wi] & 0xffffu) | (w[3][wi] << 16);
        }
        reinterpret_cast<uint2*>(&lds_vt[d * 8 + (chunk ^ (d & 7))])[within] = pk;
      }
    }
    __syncthreads();

    // S^T = K Q^T : two blocks of 32 keys
    f32x16 acc_s[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
#pragma unroll
      for (int e = 0; e < 16; ++e) acc_s[b][e] = 0.f;
      const int row = 32 * b + ql;
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const bf16x8 kf = __builtin_bit_cast(bf16x8, lds_k[row * 16 + ((2 * s + half) ^ (row & 7))]);
        acc_s[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], acc_s[b], 0, 0, 0);
      }
    }
    // scale, mask, running softmax.  Element e of block b is key kv0 + 32 b + 8 (e/4) + 4 half + e%4.
    const bool need_mask = kv0 + BKV - 1 > first_pos;
    float mx = -INFINITY;
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float s = acc_s[b][e] * c_scale;
        if (need_mask) {
          const int key = kv0 + 32 * b + 8 * (e >> 2) + 4 * half + (e & 3);
          if (key > my_pos) s = -INFINITY;
        }
        acc_s[b][e] = s;
        mx = fmaxf(mx, s);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);      // finite: key 0 is visible to every row in tile 0
    const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
    m_run = m_new;
    float psum = 0.f;
    bf16x8 pf[4];
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        f32x8 p;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          p[j] = __builtin_amdgcn_exp2f(acc_s[b][8 * u + j] - m_new);
          psum += p[j];
        }
        pf[2 * b + u] = __builtin_convertvector(p, bf16x8);
      }
    l_run = l_run * corr + psum;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc_o[i][e] *= corr;
    // O^T += V^T P
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      const int d = 32 * db + ql;
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) {
        const bf16x8 vf = __builtin_bit_cast(bf16x8, lds_vt[d * 8 + ((2 * tt + half) ^ (d & 7))]);
        acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[tt], acc_o[db], 0, 0, 0);
      }
    }
  }

  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (q_ok) {
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

template <int G>
static hipError_t launch_g(const bf16* q, const int* row_pos, const ReqTable* table, int fixed_seq, int total_rows,
                           int total_tiles, const bf16* k_pool, const bf16* v_pool, KvGeom g, bf16* out,
                           hipStream_t st) {
  dim3 grid((unsigned)total_tiles, (unsigned)g.n_kv_heads);
  attn_mfma_kernel<G><<<grid, 64 * G, 0, st>>>(q, row_pos, table, fixed_seq, total_rows, total_tiles, k_pool, v_pool,
                                               g, out);
  return hipGetLastError();
}

template <>
hipError_t launch_attention<bf16>(const bf16* q, const int* row_pos, const int* row_req, const ReqTable* table,
                                  int fixed_seq, int total_rows, int total_tiles, const bf16* k_pool,
                                  const bf16* v_pool, KvGeom g, int n_q_heads, bf16* out, hipStream_t st) {
  if (total_rows <= 0) return hipSuccess;
  const int G = n_q_heads / g.n_kv_heads;
  switch (G) {
    case 1: return launch_g<1>(q, row_pos, table, fixed_seq, total_rows, total_tiles, k_pool, v_pool, g, out, st);
    case 2: return launch_g<2>(q, row_pos, table, fixed_seq, total_rows, total_tiles, k_pool, v_pool, g, out, st);
    case 3: return launch_g<3>(q, row_pos, table, fixed_seq, total_rows, total_tiles, k_pool, v_pool, g, out, st);
    case 4: return launch_g<4>(q, row_pos, table, fixed_seq, total_rows, total_tiles, k_pool, v_pool, g, out, st);
    case 5: return launch_g<5>(q, row_pos, table, fixed_seq, total_rows, total_tiles, k_pool, v_pool, g, out, st);
    case 6: return launch_g<6>(q, row_pos, table, fixed_seq, total_rows, total_tiles, k_pool, v_pool, g, out, st);
    case 7: return launch_g<7>(q, row_pos, table, fixed_seq, total_rows, total_tiles, k_pool, v_pool, g, out, st);
    case 8: return launch_g<8>(q, row_pos, table, fixed_seq, total_rows, total_tiles, k_pool, v_pool, g, out, st);
    default:  // wider groups: one wavefront per (row, head) on the vector ALUs
      return launch_attention_simt<bf16>(q, row_pos, row_req, table, fixed_seq, total_rows, k_pool, v_pool, g,
                                         n_q_heads, out, st);
  }
}

}  // namespace rc
