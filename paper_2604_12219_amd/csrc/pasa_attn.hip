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
constexpr int kXcds = 8;  // accelerator complex dies of an MI355X

template <int D>
struct WaveState {
  bf16x8 qf[D / 16];   // Q^T fragments (B operand), fixed for the kernel
  f32x16 o[D / 32];    // O^T accumulators: o[t][reg] <-> column 32t + mfma_row(reg, h)
  float m;             // running maximum of the scaled logits, in log2 units
  float l;             // this lane's share of the running normaliser
};

// Raise the running maximum of a lane to m_new and rescale its accumulators.  Called only when some
// lane of the wave needs it (the branch around it is wave-uniform).
template <int D>
PASA_DEVICE void rescale(WaveState<D>& w, float m_new) {
  const float corr = __builtin_amdgcn_exp2f(w.m - m_new);  // exp2(-inf) = 0 on the first tile
  w.m = m_new;
  w.l *= corr;
#pragma unroll
  for (int t = 0; t < D / 32; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) w.o[t][r] *= corr;
}

// One 64-key tile: logits, online softmax, P^T fragments.  n_valid = number of valid keys (rows) in
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
  mx = half_swap_max(mx) * c;
  if (__builtin_amdgcn_ballot_w64(mx > w.m)) rescale<D>(w, fmaxf(w.m, mx));
  const float neg = -w.m;
  float sum = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    s0[r] = __builtin_amdgcn_exp2f(fmaf(s0[r], c, neg));
    s1[r] = __builtin_amdgcn_exp2f(fmaf(s1[r], c, neg));
    sum += s0[r] + s1[r];
  }
  w.l += sum;
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
// selected; blocks at or beyond nb do not exist.  On return a[r] = a_j of the block in register r
// (0 for selected or absent blocks) and pf holds the same values as P^T fragments.
template <int D>
PASA_DEVICE void approx_chunk_scores(const char* k_lds, WaveState<D>& w, float c, uint32_t word, int chunk,
                                     int nb, int block, int tail, int lane, f32x16& a, bf16x8 (&pf)[2]) {
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
  mx = half_swap_max(mx) * c;
  if (__builtin_amdgcn_ballot_w64(mx > w.m)) rescale<D>(w, fmaxf(w.m, mx));
  const float neg = -w.m;
  float sum = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    int j = 32 * chunk + mfma_row(r, h);
    z[r] = __builtin_amdgcn_exp2f(fmaf(z[r], c, neg));    // exp2(-inf) = 0 for selected / absent blocks
    sum += z[r] * (float)((j == nb - 1) ? tail : block);  // b_j a_j: this block's share of the normaliser
  }
  w.l += sum;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    pf[0][i] = (__bf16)z[i];
    pf[1][i] = (__bf16)z[8 + i];
  }
  a = z;
}

template <int D>
PASA_DEVICE void approx_chunk_pv(const char* st_lds, WaveState<D>& w, const bf16x8 (&pf)[2], int lane) {
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)  // block value sums live in rows 32..63 of the statistics tile
#pragma unroll
    for (int t = 0; t < D / 32; ++t)
      w.o[t] = mfma32(col_frag<D>(st_lds, 32 + 16 * ks, 32 * t, lane), pf[ks], w.o[t]);
}

// First-order term of one group (Eq.14), one half of the value columns: O^T[half] += (scale Hg)^T (Q^T diag(A)),
// A = sum of the chunk's a_j over the unselected blocks of the group.  h_lds holds rows
// [half*D/2, (half+1)*D/2) of (scale Hg)^T as a K-like tile (row = value column, col = key column).
template <int D>
PASA_DEVICE void first_order_half(const char* h_lds, WaveState<D>& w, float A, int half, int lane) {
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    bf16x8 qs;
#pragma unroll
    for (int i = 0; i < 8; ++i) qs[i] = (__bf16)((float)w.qf[s][i] * A);
#pragma unroll
    for (int tt = 0; tt < D / 64; ++tt) {
      const bf16x8 a = row_frag<D>(h_lds, 32 * tt, s, lane);
      if (half == 0) w.o[tt] = mfma32(a, qs, w.o[tt]);
      else w.o[D / 64 + tt] = mfma32(a, qs, w.o[D / 64 + tt]);
    }
  }
}

// Direct global -> LDS staging of a tile (no registers in between).  One instruction moves 1 KB:
// 64 lanes x 16 bytes land at consecutive LDS addresses, i.e. RPI = 1024/(2D) whole tile rows; the
// XOR swizzle of the LDS layout is applied on the global side (which chunk of its row a lane
// fetches).  Wave `wave` of NW issues instructions wave, wave + NW, ...  The swizzle pattern of a
// lane repeats every PER instructions of a wave, so PER lane offsets are kept in registers and the
// rest of the address is wave-uniform scalar arithmetic.
template <int D, int NW>
struct TileDma {
  static constexpr int CPR = D / 8;                          // 16-byte chunks per row
  static constexpr int RPI = 1024 / (2 * D);                 // rows per instruction
  static constexpr int NI = 64 / RPI / NW;                   // instructions per wave for a 64-row tile
  static constexpr int PER = (D == 128 && NW == 2) ? 2 : 1;  // (NW*RPI*PER) % 16 == 0
  static_assert((NW * RPI * PER) % 16 == 0, "swizzle period");
  uint32_t off[PER];  // byte offset of this lane's chunk for instruction i < PER, from the tile's first row

  PASA_DEVICE static int tile_row(int i, int wave, int lane) { return (i * NW + wave) * RPI + lane / CPR; }

  PASA_DEVICE void init(int64_t stride_elems, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int r = tile_row(i, wave, lane);
      off[i] = (uint32_t)(r * stride_elems * 2 + (((lane % CPR) ^ swz<D>(r)) << 4));
    }
  }
  // rows [0, ROWS) of the tile whose first row is at `base` (wave-uniform); every row is in bounds
  template <int ROWS>
  PASA_DEVICE void issue(const uint16_t* base, int64_t stride_elems, char* lds, int wave) const {
    const char* b = reinterpret_cast<const char*>(base);
#pragma unroll
    for (int i = 0; i < NI * ROWS / 64; ++i) {
      const char* bi = b + (int64_t)((i / PER) * PER * NW * RPI) * stride_elems * 2;  // uniform
      __builtin_amdgcn_global_load_lds((gbl_void*)(bi + off[i % PER]), (lds_void*)(lds + (i * NW + wave) * 1024), 16, 0, 0);
    }
  }
  // same, but tile rows at or beyond `valid` (>= 1) re-read row valid-1 (finite stand-ins for
  // rows that do not exist; the caller masks them out)
  template <int ROWS>
  PASA_DEVICE void issue_clamped(const uint16_t* base, int64_t stride_elems, int valid, char* lds, int wave,
                                 int lane) const {
    const char* b = reinterpret_cast<const char*>(base);
#pragma unroll
    for (int i = 0; i < NI * ROWS / 64; ++i) {
      const int r = tile_row(i, wave, lane);
      const int64_t o = (int64_t)min(r, valid - 1) * stride_elems * 2 + (((lane % CPR) ^ swz<D>(r)) << 4);
      __builtin_amdgcn_global_load_lds((gbl_void*)(b + o), (lds_void*)(lds + (i * NW + wave) * 1024), 16, 0, 0);
    }
  }
};

PASA_DEVICE void wait_dma_and_sync() {
  __builtin_amdgcn_s_waitcnt(0x0f70);  // vmcnt(0): this wave's direct-to-LDS loads have landed
  __syncthreads();
}

typedef __attribute__((address_space(4))) const int32_t const_i32;
typedef __attribute__((address_space(4))) const uint32_t const_u32;

template <int D, int NW, bool SPARSE>
__global__ void __launch_bounds__(NW * 64, 2) attn_kernel(AttnParams p) {
  constexpr int TILE_BYTES = 64 * 2 * D;
  // Two separate arrays (not one array indexed by parity): a pending direct-to-LDS load into one
  // must not make the compiler stall reads of the other.
  __shared__ __attribute__((aligned(1024))) char lds_x[TILE_BYTES];
  __shared__ __attribute__((aligned(1024))) char lds_y[TILE_BYTES];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ql = lane & 31, h = lane >> 5;
  // Workgroup -> (head, query tile).  The hardware deals consecutive workgroup ids round-robin to
  // the 8 XCDs (each with its own L2), so ids are decoded such that one XCD owns a contiguous run
  // of query tiles of one head and all XCDs work on the same head at the same time: neighbouring
  // query tiles select overlapping key blocks and walk them in the same (ascending) order.
  const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
  const int bh = local / p.q_tiles_per_xcd, qt = xcd * p.q_tiles_per_xcd + local % p.q_tiles_per_xcd;
  if (qt >= p.q_tiles) return;  // padding workgroup (whole workgroup leaves before any barrier)
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

  // ---- the stream of 64-row tiles that passes through LDS, alternating between lds_x and lds_y:
  //   K_0 V_0 K_1 V_1 ...            exact tiles of the selected blocks (dense: of every block)
  //   ST_0 H_{g,0} H_{g,1} ST_1 ...  per chunk of 32 key blocks: its statistics tile, then the two
  //                                  halves of every group matrix the chunk intersects
  // A tile is requested as soon as the buffer it goes to has been consumed, i.e. two tiles ahead.
  const int tiles_per_block = SPARSE ? p.block / 64 : 1;
  const int n_exact = SPARSE ? p.k_sel * tiles_per_block : (n + 63) / 64;
  const int n_chunks = (SPARSE && p.group > 0) ? p.n_chunks : 0;
  // routing lists are read through the scalar cache (constant address space): uniform, read-only
  const_i32* const idx_row = SPARSE ? (const_i32*)(p.idx + ((int64_t)bh * p.nb + qt) * p.k_sel) : nullptr;
  const_u32* const mask_row = n_chunks ? (const_u32*)(p.mask + ((int64_t)bh * p.nb + qt) * p.mask_words) : nullptr;
  const uint16_t* const st = n_chunks ? p.st + (int64_t)bh * p.n_chunks * 64 * D : nullptr;
  const uint16_t* const hg = n_chunks ? p.hg + (int64_t)bh * p.n_groups * D * D : nullptr;

  auto key_row0 = [&](int it) -> int {  // first key row of exact tile `it`
    if constexpr (SPARSE) {
      const int j = idx_row[it / tiles_per_block];
      return j * p.block + (it % tiles_per_block) * 64;
    } else {
      return it * 64;
    }
  };

  TileDma<D, NW> dma_kv, dma_st;  // lane offsets for rows of K/V (caller's stride) and of workspace tiles (stride D)
  dma_kv.init(p.stride_n, wave, lane);
  if (n_chunks) dma_st.init(D, wave, lane);

  auto stage_exact = [&](const uint16_t* src, int r0, char* lds) {
    const int valid = n - r0;
    const uint16_t* base = src + (int64_t)r0 * p.stride_n;
    if (valid >= 64) dma_kv.template issue<64>(base, p.stride_n, lds, wave);
    else if (valid >= 1) dma_kv.template issue_clamped<64>(base, p.stride_n, valid, lds, wave, lane);
    // valid <= 0: the tile does not exist (second half of a short last block); every logit of it is
    // masked and the stale, finite LDS contents meet zero weights
  };
  auto stage_stats = [&](int chunk, char* lds) { dma_st.template issue<64>(st + (int64_t)chunk * 64 * D, D, lds, wave); };
  auto stage_hg = [&](int g, int half, char* lds) {
    dma_st.template issue<D / 2>(hg + ((int64_t)g * D + half * (D / 2)) * D, D, lds, wave);
  };
  auto first_group = [&](int chunk) { return (32 * chunk) / p.group; };
  auto last_group = [&](int chunk) { return (min(32 * chunk + 32, p.nb) - 1) / p.group; };

  // ---------------- exact tiles: K in lds_x, V in lds_y ----------------
  int r0 = key_row0(0);
  stage_exact(kb, r0, lds_x);
  wait_dma_and_sync();
  stage_exact(vb, r0, lds_y);
  for (int it = 0; it < n_exact; ++it) {
    const bool more = it + 1 < n_exact;
    const int r0_next = more ? key_row0(it + 1) : 0;
    bf16x8 pf[4];
    exact_tile_scores<D>(lds_x, w, p.c, n - r0, lane, pf);
    wait_dma_and_sync();  // V tile visible to every wave; every wave is done with the K tile
    if (more) stage_exact(kb, r0_next, lds_x);
    else if (n_chunks) stage_stats(0, lds_x);
    exact_tile_pv<D>(lds_y, w, pf, lane);
    wait_dma_and_sync();  // next K (or first statistics tile) visible; every wave is done with the V tile
    if (more) stage_exact(vb, r0_next, lds_y);
    else if (n_chunks) stage_hg(first_group(0), 0, lds_y);
    r0 = r0_next;
  }

  // ---------------- grouped approximation of the unselected blocks ----------------
  // On entry of a chunk: its statistics tile is visible in `ps`, the first half of its first group
  // matrix is on its way to `pq`.  The two buffers swap roles from one chunk to the next.
  auto approx_chunk = [&](int chunk, char* ps, char* pq) {
    bf16x8 pf[2];
    f32x16 a;
    approx_chunk_scores<D>(ps, w, p.c, mask_row[chunk], chunk, p.nb, p.block, p.tail, lane, a, pf);
    approx_chunk_pv<D>(ps, w, pf, lane);
    const bool more = chunk + 1 < n_chunks;
    const int g_last = last_group(chunk);
    for (int g = first_group(chunk); g <= g_last; ++g) {
      float A = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int j = 32 * chunk + mfma_row(r, h);
        A += (j / p.group == g) ? a[r] : 0.f;
      }
      A = half_swap_sum(A);
      wait_dma_and_sync();  // first half of Hg visible in pq; ps is free
      stage_hg(g, 1, ps);
      first_order_half<D>(pq, w, A, 0, lane);
      wait_dma_and_sync();  // second half visible in ps; pq is free
      if (g < g_last) stage_hg(g + 1, 0, pq);
      else if (more) stage_stats(chunk + 1, pq);
      first_order_half<D>(ps, w, A, 1, lane);
    }
    wait_dma_and_sync();  // next statistics tile visible in pq; ps is free
    if (more) stage_hg(first_group(chunk + 1), 0, ps);
  };
  for (int chunk = 0; chunk < n_chunks; chunk += 2) {
    approx_chunk(chunk, lds_x, lds_y);
    if (chunk + 1 < n_chunks) approx_chunk(chunk + 1, lds_y, lds_x);
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
    p.q_tiles_per_xcd = (p.q_tiles + kXcds - 1) / kXcds;
    const int grid = p.bh * kXcds * p.q_tiles_per_xcd;
    if (d == 128 && p.block == 64) return launch<128, 2, true>(p, grid, stream);
    if (d == 128 && p.block == 128) return launch<128, 4, true>(p, grid, stream);
    if (d == 64 && p.block == 64) return launch<64, 2, true>(p, grid, stream);
    if (d == 64 && p.block == 128) return launch<64, 4, true>(p, grid, stream);
  } else {
    p.q_tiles = (p.n + 127) / 128;
    p.q_tiles_per_xcd = (p.q_tiles + kXcds - 1) / kXcds;
    const int grid = p.bh * kXcds * p.q_tiles_per_xcd;
    if (d == 128) return launch<128, 4, false>(p, grid, stream);
    if (d == 64) return launch<64, 4, false>(p, grid, stream);
  }
  return hipErrorInvalidValue;
}
