// Attention kernels of the PASA forward for gfx950: the exact flash-style walk over selected key
// blocks (Eq.7 first term), the grouped Taylor approximation of the unselected blocks (Eq.4, Eq.14)
// merged into the same online-softmax state, and the dense reference (Eq.1) as the special case
// "every block selected".
//
// Formulation.  Everything is computed transposed so that a lane owns one query:
//   S^T = K Q^T      (A = K rows from LDS, B = Q^T held in registers for the whole kernel)
//   O^T += V^T P^T   (A = V columns from LDS through transposing LDS reads, B = P^T cut straight
//                     from the S^T accumulator registers)
// A wave owns 32 query rows; lane (q = lane & 31, h = lane >> 5) holds for query q the logits of
// the keys 8g + 4h + r of each 32-key sub-tile (g, r = 0..3), so the row maximum and row sum are
// in-lane reductions plus one exchange with lane ^ 32.
#include "pasa_device.hpp"
#include "pasa_kernels.hpp"

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <int D>
struct WaveState {
  bf16x8 qf[D / 16];   // Q^T fragments (B operand), fixed for the kernel
  f32x16 o[D / 32];    // O^T accumulators: o[t][reg] <-> column 32t + mfma_row(reg, h)
  float m;             // running maximum of the scaled logits, in log2 units
  float l;             // this lane's share of the running normaliser
};

// One 64-key tile: logits, online softmax, accumulate.  n_valid = number of valid keys (rows) in
// the tile, may be <= 0 (nothing valid) or >= 64 (all valid).
template <int D>
PASA_DEVICE void exact_tile_scores(const char* k_lds, WaveState<D>& w, float c, int n_valid, int lane,
                                   bf16x8 (&pf)[4]) {
  const int h = lane >> 5;
  f32x16 s0 = {0}, s1 = {0};
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    s0 = mfma32(row_frag<D>(k_lds, 0, s, lane), w.qf[s], s0);
    s1 = mfma32(row_frag<D>(k_lds, 32, s, lane), w.qf[s], s1);
  }
  if (n_valid < 64) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      int key = mfma_row(r, h);
      if (key >= n_valid) s0[r] = -INFINITY;
      if (key + 32 >= n_valid) s1[r] = -INFINITY;
    }
  }
  float mx = fmaxf(s0[0], s1[0]);
#pragma unroll
  for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(s0[r], s1[r]));
  mx = half_swap_max(mx);
  const float m_new = fmaxf(w.m, mx * c);
  const float corr = __builtin_amdgcn_exp2f(w.m - m_new);
  const float neg = -m_new;
  float sum = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    s0[r] = __builtin_amdgcn_exp2f(fmaf(s0[r], c, neg));
    s1[r] = __builtin_amdgcn_exp2f(fmaf(s1[r], c, neg));
    sum += s0[r] + s1[r];
  }
  w.l = w.l * corr + sum;
  w.m = m_new;
#pragma unroll
  for (int t = 0; t < D / 32; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) w.o[t][r] *= corr;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    pf[0][i] = (__bf16)s0[i];
    pf[1][i] = (__bf16)s0[8 + i];
    pf[2][i] = (__bf16)s1[i];
    pf[3][i] = (__bf16)s1[8 + i];
  }
}

template <int D>
PASA_DEVICE void exact_tile_pv(const char* v_lds, WaveState<D>& w, const bf16x8 (&pf)[4], int lane) {
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)  // 16 keys per step: rows 16*ks ..
#pragma unroll
    for (int t = 0; t < D / 32; ++t) w.o[t] = mfma32(col_frag<D>(v_lds, 16 * ks, 32 * t, lane), pf[ks], w.o[t]);
}

// Approximation of one chunk of 32 key blocks (Eq.4 and Eq.14).  k_lds rows 0..31 hold the block-mean
// keys, v_lds rows 0..31 the block value sums.  `word` has bit x set iff block 32*chunk + x is
// selected; blocks at or beyond nb do not exist.
template <int D>
PASA_DEVICE void approx_chunk_scores(const char* k_lds, WaveState<D>& w, float c, uint32_t word, int chunk,
                                     int nb, int block, int tail, int lane, f32x16& a_out, bf16x8 (&pf)[2]) {
  const int h = lane >> 5;
  f32x16 z = {0};
#pragma unroll
  for (int s = 0; s < D / 16; ++s) z = mfma32(row_frag<D>(k_lds, 0, s, lane), w.qf[s], z);
  float mx = -INFINITY;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    int x = mfma_row(r, h), j = 32 * chunk + x;
    bool unsel = (j < nb) && !((word >> x) & 1u);
    z[r] = unsel ? z[r] : -INFINITY;
    mx = fmaxf(mx, z[r]);
  }
  mx = half_swap_max(mx);
  const float m_new = fmaxf(w.m, mx * c);
  const float corr = __builtin_amdgcn_exp2f(w.m - m_new);
  const float neg = -m_new;
  float sum = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    int j = 32 * chunk + mfma_row(r, h);
    float a = __builtin_amdgcn_exp2f(fmaf(z[r], c, neg));  // exp2(-inf) = 0 for selected / absent blocks
    z[r] = a;
    sum += a * (float)((j == nb - 1) ? tail : block);      // b_j a_j: this block's share of the normaliser
  }
  w.l = w.l * corr + sum;
  w.m = m_new;
#pragma unroll
  for (int t = 0; t < D / 32; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) w.o[t][r] *= corr;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    pf[0][i] = (__bf16)z[i];
    pf[1][i] = (__bf16)z[8 + i];
  }
  a_out = z;
}

template <int D>
PASA_DEVICE void approx_chunk_pv(const char* v_lds, WaveState<D>& w, const bf16x8 (&pf)[2], int lane) {
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
#pragma unroll
    for (int t = 0; t < D / 32; ++t) w.o[t] = mfma32(col_frag<D>(v_lds, 16 * ks, 32 * t, lane), pf[ks], w.o[t]);
}

// First-order term of one group inside a chunk: O^T += (scale Hg)^T (Q^T diag(A)), A = sum of the
// chunk's a_j over the unselected blocks that belong to the group.  hg points at the group's matrix
// in operand order: [D/32 tiles][D/16 steps][64 lanes][8] bf16 (see the statistics kernel).
template <int D>
PASA_DEVICE void first_order(const uint16_t* hg, WaveState<D>& w, float A, int lane) {
  bf16x8 qs[D / 16];
#pragma unroll
  for (int s = 0; s < D / 16; ++s)
#pragma unroll
    for (int i = 0; i < 8; ++i) qs[s][i] = (__bf16)((float)w.qf[s][i] * A);
  const uint4* frag = reinterpret_cast<const uint4*>(hg) + lane;
#pragma unroll
  for (int t = 0; t < D / 32; ++t)
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      uint4 raw = frag[(t * (D / 16) + s) * 64];
      w.o[t] = mfma32(__builtin_bit_cast(bf16x8, raw), qs[s], w.o[t]);
    }
}

template <int D, int NW, bool SPARSE>
__global__ void __launch_bounds__(NW * 64, 2) attn_kernel(AttnParams p) {
  constexpr int T = NW * 64;
  constexpr int TILE_BYTES = 64 * 2 * D;
  __shared__ __attribute__((aligned(16))) char smem[2 * TILE_BYTES];
  char* const k_lds = smem;
  char* const v_lds = smem + TILE_BYTES;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ql = lane & 31, h = lane >> 5;
  const int bh = blockIdx.x / p.q_tiles, qt = blockIdx.x % p.q_tiles;
  const int64_t head_off = (int64_t)(bh / p.H) * p.stride_b + (int64_t)(bh % p.H) * p.stride_h;
  const uint16_t* const qb = p.q + head_off;
  const uint16_t* const kb = p.k + head_off;
  const uint16_t* const vb = p.v + head_off;
  const int n = p.n;
  const int q_row = qt * (NW * 32) + wave * 32 + ql;

  WaveState<D> w;
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    uint4 raw = {0u, 0u, 0u, 0u};
    if (q_row < n) raw = *reinterpret_cast<const uint4*>(qb + (int64_t)q_row * p.stride_n + 16 * s + 8 * h);
    w.qf[s] = __builtin_bit_cast(bf16x8, raw);
  }
#pragma unroll
  for (int t = 0; t < D / 32; ++t) w.o[t] = f32x16{0};
  w.m = -INFINITY;
  w.l = 0.f;

  // ---- the item list: exact 64-key tiles first, then chunks of 32 block statistics ----
  const int tiles_per_block = SPARSE ? p.block / 64 : 1;
  const int n_exact = SPARSE ? p.k_sel * tiles_per_block : (n + 63) / 64;
  const int n_chunks = (SPARSE && p.group > 0) ? (p.nb + 31) / 32 : 0;
  const int n_items = n_exact + n_chunks;
  const int32_t* const idx_row = SPARSE ? p.idx + ((int64_t)bh * p.nb + qt) * p.k_sel : nullptr;
  const uint32_t* const mask_row = (SPARSE && p.group > 0) ? p.mask + ((int64_t)bh * p.nb + qt) * p.mask_words : nullptr;
  const uint16_t* const kbar = SPARSE ? p.kbar + (int64_t)bh * p.nb * D : nullptr;
  const uint16_t* const vsum = SPARSE ? p.vs + (int64_t)bh * p.nb * D : nullptr;

  auto key_row0 = [&](int it) -> int {  // first key row of exact item `it`
    if constexpr (SPARSE) {
      int j = idx_row[it / tiles_per_block];
      return j * p.block + (it % tiles_per_block) * 64;
    } else {
      return it * 64;
    }
  };

  TileStage<D, T> st;
  auto load_k = [&](int it) {
    if (it < n_exact) st.load(kb, p.stride_n, key_row0(it), 64, n, tid);
    else st.load(kbar, D, 32 * (it - n_exact), 32, p.nb, tid);
  };
  auto load_v = [&](int it) {
    if (it < n_exact) st.load(vb, p.stride_n, key_row0(it), 64, n, tid);
    else st.load(vsum, D, 32 * (it - n_exact), 32, p.nb, tid);
  };
  auto rows_of = [&](int it) { return it < n_exact ? 64 : 32; };

  load_k(0);
  st.store(k_lds, rows_of(0), tid);
  load_v(0);
  st.store(v_lds, rows_of(0), tid);
  __syncthreads();

  for (int it = 0; it < n_items; ++it) {
    const bool has_next = it + 1 < n_items;
    if (has_next) load_k(it + 1);
    if (it < n_exact) {
      bf16x8 pf[4];
      const int n_valid = n - key_row0(it);
      exact_tile_scores<D>(k_lds, w, p.c, n_valid, lane, pf);
      __syncthreads();  // every wave has read the K tile
      if (has_next) {
        st.store(k_lds, rows_of(it + 1), tid);
        load_v(it + 1);
      }
      exact_tile_pv<D>(v_lds, w, pf, lane);
    } else {
      const int chunk = it - n_exact;
      const uint32_t word = mask_row[chunk];
      bf16x8 pf[2];
      f32x16 a;
      approx_chunk_scores<D>(k_lds, w, p.c, word, chunk, p.nb, p.block, p.tail, lane, a, pf);
      __syncthreads();
      if (has_next) {
        st.store(k_lds, rows_of(it + 1), tid);
        load_v(it + 1);
      }
      approx_chunk_pv<D>(v_lds, w, pf, lane);
      // first-order term, one pass per group that intersects this chunk
      const int j_lo = 32 * chunk, j_hi = min(j_lo + 32, p.nb);
      for (int g = j_lo / p.group; g <= (j_hi - 1) / p.group; ++g) {
        float A = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int j = j_lo + mfma_row(r, h);
          A += (j / p.group == g) ? a[r] : 0.f;
        }
        A = half_swap_sum(A);
        first_order<D>(p.hg + ((int64_t)bh * p.n_groups + g) * D * D, w, A, lane);
      }
    }
    __syncthreads();  // every wave has read the V tile
    if (has_next) st.store(v_lds, rows_of(it + 1), tid);
    __syncthreads();  // next K and V tiles are visible
  }

  // ---- epilogue: normalise and write ----
  const float l_tot = half_swap_sum(w.l);
  const float inv = 1.0f / l_tot;
  if (q_row < n) {
    uint16_t* orow = p.o + head_off + (int64_t)q_row * p.stride_n;
#pragma unroll
    for (int t = 0; t < D / 32; ++t)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
        bf16x4 ov;
#pragma unroll
        for (int r = 0; r < 4; ++r) ov[r] = (__bf16)(w.o[t][4 * g + r] * inv);
        *reinterpret_cast<bf16x4*>(orow + 32 * t + 8 * g + 4 * h) = ov;
      }
    if (p.lse && h == 0) p.lse[(int64_t)bh * n + q_row] = (w.m + __builtin_amdgcn_logf(l_tot)) * kLn2;
  }
}

template <int D, int NW, bool SPARSE>
hipError_t launch(const AttnParams& p, int grid, hipStream_t stream) {
  hipLaunchKernelGGL((attn_kernel<D, NW, SPARSE>), dim3(grid), dim3(NW * 64), 0, stream, p);
  return hipGetLastError();
}

}  // namespace

hipError_t pasa_launch_attn(AttnParams p, bool sparse, int d, hipStream_t stream) {
  p.c = p.scale * kLog2e;
  if (sparse) {
    p.q_tiles = p.nb;  // one workgroup per query block
    const int grid = p.bh * p.q_tiles;
    if (d == 128 && p.block == 64) return launch<128, 2, true>(p, grid, stream);
    if (d == 128 && p.block == 128) return launch<128, 4, true>(p, grid, stream);
    if (d == 64 && p.block == 64) return launch<64, 2, true>(p, grid, stream);
    if (d == 64 && p.block == 128) return launch<64, 4, true>(p, grid, stream);
  } else {
    p.q_tiles = (p.n + 127) / 128;
    const int grid = p.bh * p.q_tiles;
    if (d == 128) return launch<128, 4, false>(p, grid, stream);
    if (d == 64) return launch<64, 4, false>(p, grid, stream);
  }
  return hipErrorInvalidValue;
}
