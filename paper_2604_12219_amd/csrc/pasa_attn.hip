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
//
// Work decomposition.  A workgroup is 4 waves = 128 query rows: one query block of 128 tokens, or
// TWO ADJACENT query blocks of 64 tokens (waves 0,1 and waves 2,3).  In the second case the
// workgroup walks the UNION of the two ascending block lists; a tile is staged in LDS once and each
// wave pair computes on it only if its own list contains the block.  Adjacent query blocks of a
// video select heavily overlapping key blocks, so this cuts the K/V traffic per query block.
//
// Key-range slicing (sparse path, long sequences).  L2 misses of all XCDs share one fabric whose read
// bandwidth is far below what the eight L2s deliver on hits, and one head's K and V are much larger
// than one L2.  So the key range is cut into slices that fit an L2; workgroups whose id is congruent
// to x modulo 8 run on XCD x and walk only slice x (+8, +16, ...) of every query tile.  Each slice of
// K and V is then fetched from memory once per head and XCD and hit in L2 afterwards.  Every
// workgroup leaves an unnormalised partial result (running maximum, normaliser share, numerator),
// and a small second kernel merges the partial results of a row.
//
// Data movement.  All tiles (K, V, block statistics, group matrices) are 64-row tiles that stream
// through a ring of four LDS buffers by direct global->LDS loads, requested three tiles ahead of
// their use; one workgroup barrier per tile.
#include "pasa_device.hpp"
#include "pasa_kernels.hpp"
#include "pasa_mfma_pipes.hpp"
#include <stdlib.h>

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kXcds = 8;    // accelerator complex dies of an MI355X, each with its own L2
constexpr int kWaves = 4;   // waves per workgroup
constexpr int kRing = 4;    // LDS tile buffers
constexpr int kAhead = 3;   // a tile is requested this many tiles before it is consumed
constexpr int kNoBlock = 0x7fffffff;
#ifdef PASA_DEBUG_MODES
constexpr bool kDebugModes = true;   // timing experiments: results are wrong on purpose
#else
constexpr bool kDebugModes = false;
#endif
#ifdef PASA_PROFILE_PHASES
constexpr bool kProfile = true;      // per-phase cycle counts of the exact loop into AttnParams::prof
#else
constexpr bool kProfile = false;
#endif
PASA_DEVICE uint32_t clock32() { return (uint32_t)__builtin_amdgcn_s_memtime(); }

typedef __attribute__((address_space(4))) const int32_t const_i32;
typedef __attribute__((address_space(4))) const uint32_t const_u32;

template <int D>
struct WaveState {
  bf16x8 qf[D / 16];   // Q^T fragments (B operand), fixed for the kernel
  f32x16 o[D / 32];    // O^T accumulators: o[t][reg] <-> column 32t + mfma_row(reg, h)
  float m;             // running maximum of the scaled logits, in log2 units
  float l;             // this lane's share of the running normaliser
};

// Per-lane byte offsets of the MFMA operand fetches inside a 64-row LDS tile, computed once.  The XOR
// swizzle makes them lane-dependent, but the contraction step of a row fragment and the value-column
// tile of a column fragment enter the address as an XOR with a constant, and a multiple of 16 rows as
// an added constant (see pasa_mfma_pipes.hpp), so three registers serve every fetch of every tile.
template <int D>
struct LaneOffsets {
  uint32_t k;     // row fragment of rows 0..31, contraction step 0
  uint32_t v[2];  // column fragment of rows 0..15, value columns 0..31; [1]: the rows 8 further down
  PASA_DEVICE void init(int lane) {
    const int i = lane & 15, half16 = (lane >> 4) & 1, h = lane >> 5;
    k = (uint32_t)lds_chunk_off<D>(lane & 31, h);
    const int row = 4 * h + (i >> 2), col = 16 * half16 + 4 * (i & 3);
    v[0] = (uint32_t)(lds_chunk_off<D>(row, col >> 3) + (col & 7) * 2);
    v[1] = (uint32_t)(lds_chunk_off<D>(row + 8, col >> 3) + (col & 7) * 2);
  }
};

PASA_DEVICE float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

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

// Online softmax of one 64-key tile whose logits S^T = K Q^T are in s0 (keys 0..31) and s1 (keys 32..63):
// updates the running maximum and normaliser and leaves the P^T fragments.  n_valid = number of valid
// keys (rows) in the tile, may be <= 0 (nothing valid) or >= 64 (all valid).
template <int D>
PASA_DEVICE void exact_tile_softmax(f32x16& s0, f32x16& s1, WaveState<D>& w, float c, int n_valid, int lane,
                                    bf16x8 (&pf)[4]) {
  if (n_valid < 64) {
    const int nv = n_valid - 4 * (lane >> 5);  // key 8g + 4h + r is valid iff 8g + r < n_valid - 4h
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = mfma_row(r, 0);
      if (key >= nv) s0[r] = -INFINITY;
      if (key + 32 >= nv) s1[r] = -INFINITY;
    }
  }
  float mx = fmaxf(s0[0], s1[0]);
#pragma unroll
  for (int r = 1; r < 16; ++r) mx = max3(mx, s0[r], s1[r]);
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

// Zeroth-order part of one chunk of 32 key blocks (Eq.4).  Rows 0..31 of the statistics tile hold
// the block-mean keys, rows 32..63 the block value sums.  `word` has bit x set iff block
// 32*chunk + x is selected; blocks at or beyond nb do not exist.  On return a[r] = a_j of the block
// in register r (0 for selected or absent blocks).
template <int D>
PASA_DEVICE void approx_chunk_zeroth(uint32_t tile, const LaneOffsets<D>& lo, WaveState<D>& w, float c, uint32_t word,
                                     int chunk, int nb, int block, int tail, int lane, f32x16& a) {
  const int h = lane >> 5;
  f32x16 z, z1;
  pipes::rows32_x_q(tile + lo.k, w.qf, z, z1);
  float mx = -INFINITY;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    int x = mfma_row(r, h), j = 32 * chunk + x;
    bool unsel = (j < nb) && !((word >> x) & 1u);
    z[r] = unsel ? z[r] + z1[r] : -INFINITY;
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
  bf16x8 pf[2];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    pf[0][i] = (__bf16)z[i];
    pf[1][i] = (__bf16)z[8 + i];
  }
  pipes::cols_x_p32_hi(tile + lo.v[0], tile + lo.v[1], pf, w.o);
  a = z;
}

// First-order term of one group (Eq.14), 64 value columns at a time: O^T[part] += ((scale Hg)^T Q^T) diag(A),
// A = sum of the chunk's a_j over the unselected blocks of the group.  The tile holds rows
// [64*part, 64*part + 64) of (scale Hg)^T as a K-like tile (row = value column, col = key column).
template <int D, int PART>
PASA_DEVICE void first_order_part(uint32_t tile, const LaneOffsets<D>& lo, WaveState<D>& w, float A) {
  // q~ Hg for this lane's query (a lane owns one query, so its group weight A is a per-lane scalar
  // that multiplies the finished product)
  f32x16 w0, w1;
  pipes::rows_x_q(tile + lo.k, w.qf, w0, w1);
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    w.o[2 * PART][r] = fmaf(A, w0[r], w.o[2 * PART][r]);
    w.o[2 * PART + 1][r] = fmaf(A, w1[r], w.o[2 * PART + 1][r]);
  }
}

// ---- direct global -> LDS tile loads ------------------------------------------------------------
// One instruction moves 1 KB: 64 lanes x 16 bytes land at consecutive LDS addresses starting at M0,
// i.e. RPI = 1024/(2D) whole tile rows; the XOR swizzle of the LDS layout is applied on the global
// side (which 16-byte chunk of its row a lane fetches).  Wave w issues instruction slots w, w+4, ...
// The loads are written as inline assembly so that the compiler's wait-count insertion does not see
// them (it would serialise every LDS read behind all pending loads); ordering is by the counted
// waits in ring_barrier().  A wait count the compiler derives for its own loads can only become
// stricter by loads it does not know about (loads complete in issue order), never too weak.
PASA_DEVICE void dma_1k(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(sbase)
               : "memory", "m0");
}

template <int D>
struct TileDma {
  static constexpr int CPR = D / 8;                 // 16-byte chunks per row
  static constexpr int RPI = 1024 / (2 * D);        // rows per instruction
  static constexpr int NI = 64 / RPI / kWaves;      // instructions per wave and tile
  static_assert((kWaves * RPI) % 16 == 0, "a lane's swizzle must not change between its instructions");

  PASA_DEVICE static int tile_row(int i, int wave, int lane) { return (i * kWaves + wave) * RPI + lane / CPR; }
  PASA_DEVICE static uint32_t chunk_off(int row, int lane) { return (uint32_t)(((lane % CPR) ^ swz<D>(row)) << 4); }

  // per-lane byte offsets of the lane's chunk in each of the wave's NI instructions, for a given row
  // stride (a lane's swizzle is the same in all of them; the rows are kWaves*RPI apart)
  PASA_DEVICE static void lane_offsets(int64_t stride_elems, int wave, int lane, uint32_t (&voff)[NI]) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int r = tile_row(i, wave, lane);
      voff[i] = (uint32_t)(r * stride_elems * 2) + chunk_off(r, lane);
    }
  }
  // all 64 rows are in bounds.  base: wave-uniform address of the tile's first row; lds_wave: LDS
  // address of the slot plus wave*1024.
  PASA_DEVICE static void issue(const void* base, const uint32_t (&voff)[NI], uint32_t lds_wave) {
#pragma unroll
    for (int i = 0; i < NI; ++i) dma_1k(base, voff[i], lds_wave + (uint32_t)(i * kWaves * 1024));
  }
  // tile rows at or beyond `valid` (>= 1) re-read row valid-1 of the tile (finite stand-ins for rows
  // that do not exist; the caller masks them out).
  PASA_DEVICE static void issue_clamped(const uint16_t* base, int64_t stride_elems, int valid, uint32_t lds, int wave,
                                        int lane) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int r = tile_row(i, wave, lane);
      const uint32_t voff = (uint32_t)(min(r, valid - 1) * stride_elems * 2) + chunk_off(r, lane);
      dma_1k(base, voff, lds + (uint32_t)((i * kWaves + wave) * 1024));
    }
  }
};

// Wait until at most `newer` tiles requested after the one about to be read are still in flight
// (each wave issues NI loads per tile), and until this wave's LDS reads of the previous tile have
// returned; then meet the other waves.  After the barrier the tile is complete in LDS and the buffer
// of the previous tile may be overwritten.
template <int NI>
PASA_DEVICE void ring_barrier(int newer) {
  if (newer >= 2) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * NI) : "memory");
  else if (newer == 1) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(NI) : "memory");
  else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ---- the ascending walk over the union of (up to) two block lists --------------------------------
struct UnionWalk {
  const_i32* la;
  const_i32* lb;
  int k_a, k_b;        // list lengths (0 = list absent)
  int ia, ib, va, vb;  // cursors and the block ids under them (kNoBlock when exhausted)
  int sub;             // 64-key tile within the current block
  PASA_DEVICE void init(const_i32* a, int ka, const_i32* b, int kb) {
    la = a; lb = b; k_a = ka; k_b = kb; ia = ib = sub = 0;
    va = ka > 0 ? a[0] : kNoBlock;
    vb = kb > 0 ? b[0] : kNoBlock;
  }
  PASA_DEVICE bool done() const { return va == kNoBlock && vb == kNoBlock; }
  PASA_DEVICE int block() const { return min(va, vb); }  // current block id
  PASA_DEVICE bool in_a() const { return va <= vb; }      // ... and which lists contain it
  PASA_DEVICE bool in_b() const { return vb <= va; }
  PASA_DEVICE void advance(int tiles_per_block) {
    if (++sub < tiles_per_block) return;
    sub = 0;
    const int j = min(va, vb);
    if (va == j) { ++ia; va = ia < k_a ? la[ia] : kNoBlock; }
    if (vb == j) { ++ib; vb = ib < k_b ? lb[ib] : kNoBlock; }
  }
};

// MULTI: the group has fewer than 32 blocks, so a chunk of 32 blocks intersects several groups and
// the per-block weights of a chunk have to be kept until all of its group matrices have passed.
template <int D, bool SPARSE, bool MULTI>
__global__ void __launch_bounds__(kWaves * 64, 2) attn_kernel(AttnParams p) {
  constexpr int TILE_BYTES = 64 * 2 * D;
  constexpr int NI = TileDma<D>::NI;
  constexpr int HPARTS = D / 64;  // 64-row tiles per group matrix
  __shared__ __attribute__((aligned(1024))) char ring[kRing * TILE_BYTES];

  __shared__ int s_item;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ql = lane & 31, h = lane >> 5;
  const uint32_t ring_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)ring;
  LaneOffsets<D> lo;
  lo.init(lane);
  uint32_t voff_kv[NI], voff_ws[NI];  // lane offsets of the tile loads: rows of K/V (caller's stride), workspace tiles
  TileDma<D>::lane_offsets(p.stride_n, wave, lane, voff_kv);
  TileDma<D>::lane_offsets(D, wave, lane, voff_ws);
  const uint32_t ring_wave = ring_base + (uint32_t)(wave * 1024);
  const uint32_t row_bytes = (uint32_t)(p.stride_n * 2);
  int issued = 0;  // tiles requested so far; tile i goes to ring slot i & 3 (keeps counting across work items)
  int it = 0;      // tiles consumed so far
  const bool persistent = p.n_slices > 1;
  int xcd = blockIdx.x % kXcds;
  if (persistent) {  // ask the hardware which XCD this workgroup really runs on
    unsigned id;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(id));
    xcd = (int)(id & 15u) % kXcds;
  }

  // Work items.  Without key-range slicing a workgroup handles exactly one (head, query tile): the
  // hardware deals consecutive workgroup ids round-robin to the 8 XCDs, and ids are decoded such
  // that one XCD owns a contiguous run of query tiles of one head and all XCDs work on the same head
  // at the same time.  With slicing the kernel is persistent: two workgroups per CU, each taking
  // (head, round, query tile) items from the queue of the XCD it runs on until the queue is empty;
  // XCD x walks key slice x + 8 * round.  (A plain grid would not do: workgroups are dispatched in
  // id order, ids are bound to XCDs, and the items of one XCD take very different times -- a
  // query tile selects many more blocks from the slice it lies in -- so one busy XCD would hold up
  // the dispatch to all the others.)
  for (;;) {
  int bh, qt, slice = 0;
  if (persistent) {
    if (tid == 0) s_item = (int)atomicAdd(p.queue + xcd, 1u);
    __syncthreads();
    const int item = s_item;
    __syncthreads();  // everyone has read s_item before it can be written again
    if (item >= p.items_per_xcd) return;  // queue empty: every wave of the workgroup leaves here
    const int rounds = p.n_slices / kXcds;
    const int hr = item / p.q_tiles;
    slice = (hr % rounds) * kXcds + xcd;
    bh = hr / rounds;
    // start each slice's sweep over the query tiles at the tiles that lie in the slice itself
    qt = (int)((item % p.q_tiles + (int64_t)slice * p.q_tiles / p.n_slices) % p.q_tiles);
  } else {
    const int local = blockIdx.x / kXcds;
    bh = local / p.q_tiles_per_xcd;
    qt = xcd * p.q_tiles_per_xcd + local % p.q_tiles_per_xcd;
    if (qt >= p.q_tiles) return;  // padding workgroup (the whole workgroup leaves before any barrier)
  }
  const int64_t head_off = (int64_t)(bh / p.H) * p.stride_b + (int64_t)(bh % p.H) * p.stride_h;
  const uint16_t* const qb = p.q + head_off;
  const uint16_t* const kb = p.k + head_off;
  const uint16_t* const vb = p.v + head_off;
  const int n = p.n;
  const int q_row = qt * 128 + wave * 32 + ql;

  WaveState<D> w;
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    uint4 raw = {0u, 0u, 0u, 0u};
    if (q_row < n && !(kDebugModes && p.debug_mode == 4)) raw = *reinterpret_cast<const uint4*>(qb + (int64_t)q_row * p.stride_n + 16 * s + 8 * h);
    w.qf[s] = __builtin_bit_cast(bf16x8, raw);
  }
  // Have the query loads land here.  Otherwise the compiler, which cannot see the tile loads written in
  // assembly, waits for "all loads" at the first use of Q inside the tile loop, in every iteration, and
  // so also for the tiles that were requested just before -- the prefetch would never overlap the math.
#pragma unroll
  for (int s = 0; s < D / 16; ++s) asm volatile("" : "+v"(w.qf[s]));
#pragma unroll
  for (int t = 0; t < D / 32; ++t) w.o[t] = f32x16{0};
  w.m = -INFINITY;
  w.l = 0.f;

  // ---- which query block this wave belongs to, and the block lists of the workgroup ----
  const int qpw = SPARSE ? 128 / p.block : 1;             // query blocks per workgroup: 1 or 2
  const bool second = SPARSE && qpw == 2 && (wave >> 1);  // this wave works for the second list
  const int my_qb = SPARSE ? qt * qpw + (second ? 1 : 0) : 0;
  const bool qb_exists = !SPARSE || my_qb < p.nb;         // the second block of the last pair may not exist
  const int tiles_per_block = SPARSE ? p.block / 64 : 1;
  const int n_dense_tiles = (n + 63) / 64;
  const bool approx_on = SPARSE && p.group > 0;
  const uint16_t* const st = approx_on ? p.st + (int64_t)bh * p.n_chunks * 64 * D : nullptr;
  const uint16_t* const hg = approx_on ? p.hg + (int64_t)bh * p.n_groups * D * D : nullptr;
  const_u32* const mask_row =
      (approx_on && qb_exists) ? (const_u32*)(p.mask + ((int64_t)bh * p.nb + my_qb) * p.mask_words) : nullptr;

  // chunk range of this workgroup's slice, and for each list the entries that fall into it: their
  // number and the position of the first one are popcounts over the selection bitmap
  const int c_lo = SPARSE ? (int)((int64_t)slice * p.n_chunks / p.n_slices) : 0;
  const int c_hi = SPARSE ? (int)((int64_t)(slice + 1) * p.n_chunks / p.n_slices) : 0;
  int first_a = 0, count_a = SPARSE ? p.k_sel : 0, first_b = 0, count_b = 0;
  if constexpr (SPARSE) {
    const bool has_b = qpw == 2 && qt * 2 + 1 < p.nb;
    count_b = has_b ? p.k_sel : 0;
    if (p.n_slices > 1) {
      auto bits_in = [&](const uint32_t* row, int w0, int w1) -> int {  // wave-uniform result
        int acc = 0;
        for (int x = w0 + lane; x < w1; x += 64) acc += __popc(row[x]);
#pragma unroll
        for (int sh = 32; sh >= 1; sh >>= 1) acc += __shfl_xor(acc, sh);
        return __builtin_amdgcn_readfirstlane(acc);
      };
      const uint32_t* ma = p.mask + ((int64_t)bh * p.nb + (int64_t)qt * qpw) * p.mask_words;
      first_a = bits_in(ma, 0, c_lo);
      count_a = bits_in(ma, c_lo, c_hi);
      if (has_b) {
        first_b = bits_in(ma + p.mask_words, 0, c_lo);
        count_b = bits_in(ma + p.mask_words, c_lo, c_hi);
      }
    }
  }
  auto make_walk = [&]() {
    UnionWalk u;
    if constexpr (SPARSE) {
      const_i32* base = (const_i32*)(p.idx + ((int64_t)bh * p.nb + (int64_t)qt * qpw) * p.k_sel);
      u.init(base + first_a, count_a, base + p.k_sel + first_b, count_b);
    } else {
      u.init(nullptr, 0, nullptr, 0);
    }
    return u;
  };
  auto first_group = [&](int chunk) { return (32 * chunk) / p.group; };
  auto last_group = [&](int chunk) { return (min(32 * chunk + 32, p.nb) - 1) / p.group; };

  // ---- the producers.  A tile that is requested goes to ring slot `issued & 3`; the consumer learns what it
  // is from a descriptor:
  //   bits 0-2 kind; bit 3 / bit 4: the block is in the first / second list;
  //   K tiles:           bits 5-11  number of valid rows, clamped to [0, 64]  (its V tile follows it)
  //   statistics, Hg:    bits 5-12  chunk, bits 14-25 group
  enum : uint32_t { kEnd = 0, kKTile = 1, kStats = 3, kHPart = 4 };
  auto slot = [&](int i) -> uint32_t { return ring_base + (uint32_t)((i & (kRing - 1)) * TILE_BYTES); };
  auto slot_wave = [&](int i) -> uint32_t { return ring_wave + (uint32_t)((i & (kRing - 1)) * TILE_BYTES); };

  // exact phase: requests the K tile and the V tile of the next step of the walk into the next two slots
  UnionWalk pw = make_walk();
  int p_dense = 0;  // dense: next tile
  auto produce_pair = [&]() -> uint32_t {
    if (SPARSE ? pw.done() : (p_dense >= n_dense_tiles)) return kEnd;
    if (kDebugModes && p.debug_mode == 1 && issued >= 2) { issued += 2; if constexpr (SPARSE) pw.advance(tiles_per_block); else ++p_dense; return kKTile | 8u | 16u | (64u << 5); }
    const int r0 = SPARSE ? pw.block() * p.block + pw.sub * 64 : p_dense * 64;
    const int valid = n - r0;
    uint32_t desc = kKTile | ((uint32_t)min(max(valid, 0), 64) << 5);
    if constexpr (SPARSE) desc |= (pw.in_a() ? 8u : 0u) | (pw.in_b() ? 16u : 0u);
    else desc |= 8u;
    if (valid >= 64) {
      const uint32_t off = (uint32_t)r0 * row_bytes;
      TileDma<D>::issue(reinterpret_cast<const char*>(kb) + off, voff_kv, slot_wave(issued));
      TileDma<D>::issue(reinterpret_cast<const char*>(vb) + off, voff_kv, slot_wave(issued + 1));
    } else {  // the ragged last tile, or the tile after it in a 128-token block: rows past the end re-read the last row
      const int rr = valid >= 1 ? r0 : n - 1, vv = valid >= 1 ? valid : 1;
      TileDma<D>::issue_clamped(kb + (int64_t)rr * p.stride_n, p.stride_n, vv, slot(issued), wave, lane);
      TileDma<D>::issue_clamped(vb + (int64_t)rr * p.stride_n, p.stride_n, vv, slot(issued + 1), wave, lane);
    }
    issued += 2;
    if constexpr (SPARSE) pw.advance(tiles_per_block);
    else ++p_dense;
    return desc;
  };

  // approximation phase: requests the next tile: per chunk its statistics tile, then the HPARTS tiles of
  // every group matrix the chunk intersects
  const int c_end = approx_on ? c_hi : 0;        // chunks [c_lo, c_end) are approximated by this workgroup
  int p_chunk = c_lo, p_group = 0, p_part = -1;  // p_part == -1: statistics tile next
  auto produce_approx = [&]() -> uint32_t {
    if (p_chunk >= c_end) return kEnd;
    uint32_t desc;
    if (p_part < 0) {
      TileDma<D>::issue(st + (int64_t)p_chunk * 64 * D, voff_ws, slot_wave(issued));
      desc = kStats | ((uint32_t)p_chunk << 5);
      p_group = first_group(p_chunk);
      p_part = 0;
    } else {
      TileDma<D>::issue(hg + ((int64_t)p_group * D + 64 * p_part) * D, voff_ws, slot_wave(issued));
      desc = kHPart | ((uint32_t)p_chunk << 5) | ((uint32_t)p_group << 14);
      if (++p_part == HPARTS) {
        p_part = 0;
        if (++p_group > last_group(p_chunk)) { ++p_chunk; p_part = -1; }
      }
    }
    ++issued;
    return desc;
  };

  // ---- the consumer: tile `it` of the stream lives in ring slot it & 3 ----
  uint32_t d0 = kEnd, d1 = kEnd, d2 = kEnd;  // approximation tiles requested but not yet consumed, in order

  // ---------------- exact tiles: one barrier per (K tile, V tile) pair ----------------
  // While a pair is being consumed the next pair (or the head of the approximation stream) is on its
  // way into the other two ring slots.
  uint32_t prof[6] = {0, 0, 0, 0, 0, 0};  // cycles: wait, scores, produce, PV; steps mine, steps not mine
  const uint64_t wg_t0 = kProfile ? __builtin_amdgcn_s_memtime() : 0ull;
  const uint64_t wg_r0 = kProfile ? __builtin_amdgcn_s_memrealtime() : 0ull;
  uint32_t dk = produce_pair();
  if (dk == kEnd) { d0 = produce_approx(); d1 = produce_approx(); }
#pragma unroll 1
  while (dk != kEnd) {
    bf16x8 pf[4];  // P^T of the tile
    const uint32_t t0 = kProfile ? clock32() : 0u;
    ring_barrier<NI>(0);  // the pair has landed; every wave is done with the previous pair
    const uint32_t tb = kProfile ? clock32() : 0u;
    const uint32_t cur = dk;
    dk = produce_pair();
    if (dk == kEnd) { d0 = produce_approx(); d1 = produce_approx(); }
    const bool mine = qb_exists && ((cur >> (second ? 4 : 3)) & 1u) && !(kDebugModes && p.debug_mode == 2);
    const uint32_t t1 = kProfile ? clock32() : 0u;
    if (mine) {
      f32x16 s0, s1;
      pipes::rows_x_q(slot(it) + lo.k, w.qf, s0, s1);
      exact_tile_softmax<D>(s0, s1, w, p.c, (int)((cur >> 5) & 127u), lane, pf);
    }
    const uint32_t t2 = kProfile ? clock32() : 0u;
    if (mine) pipes::cols_x_p64(slot(it + 1) + lo.v[0], slot(it + 1) + lo.v[1], pf, w.o);
    it += 2;
    if (kProfile) {
      const uint32_t t4 = clock32();
      prof[0] += tb - t0; prof[2] += t1 - tb; prof[1] += t2 - t1; prof[3] += t4 - t2;
      prof[mine ? 4 : 5] += 1;
    }
  }
  if (kProfile && p.prof && lane == 0) {
    for (int x = 0; x < 6; ++x) atomicAdd(p.prof + wave * 8 + x, (unsigned long long)prof[x]);
    atomicAdd(p.prof + wave * 8 + 6, (unsigned long long)(__builtin_amdgcn_s_memtime() - wg_t0));
    atomicAdd(p.prof + wave * 8 + 7, (unsigned long long)(__builtin_amdgcn_s_memrealtime() - wg_r0));
  }

  // Moves on to the next tile of the approximation stream: waits for it, meets the other waves (after
  // which the slots of all earlier tiles are free) and tops the ring up to three tiles ahead.
  // Returns the descriptor of the tile to consume (slot(it)).
  auto next_tile = [&]() -> uint32_t {
    const uint32_t cur = d0;
    ring_barrier<NI>((d1 != kEnd ? 1 : 0) + (d2 != kEnd ? 1 : 0));
    d0 = d1;
    d1 = d2;
    d2 = kEnd;
    if (d0 == kEnd) d0 = produce_approx();
    if (d1 == kEnd && d0 != kEnd) d1 = produce_approx();
    if (d2 == kEnd && d1 != kEnd) d2 = produce_approx();
    return cur;
  };

  // ---------------- grouped approximation of the unselected blocks ----------------
  // per chunk of 32 key blocks: its statistics tile, then for every group it intersects the HPARTS
  // tiles of the group matrix
#pragma unroll 1
  while (d0 != kEnd) {
    f32x16 a;  // a_j of the chunk
    const uint32_t cur = next_tile();
    const int chunk = (int)((cur >> 5) & 255u);
    if (qb_exists) approx_chunk_zeroth<D>(slot(it), lo, w, p.c, mask_row[chunk], chunk, p.nb, p.block, p.tail, lane, a);
    ++it;
    float A = 0.f;
    if constexpr (!MULTI) {  // the whole chunk belongs to one group
      if (qb_exists) {
#pragma unroll
        for (int r = 0; r < 16; ++r) A += a[r];
        A = half_swap_sum(A);
      }
    }
#pragma unroll 1
    while ((d0 & 7u) == kHPart) {
      if constexpr (MULTI) {
        const int g = (int)((d0 >> 14) & 4095u);
        A = 0.f;
        if (qb_exists) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = 32 * chunk + mfma_row(r, h);
            A += (j / p.group == g) ? a[r] : 0.f;
          }
          A = half_swap_sum(A);
        }
      }
      next_tile();
      if (qb_exists) first_order_part<D, 0>(slot(it), lo, w, A);
      ++it;
      if constexpr (D == 128) {
        next_tile();
        if (qb_exists) first_order_part<D, 1>(slot(it), lo, w, A);
        ++it;
      }
    }
  }

  // ---- epilogue ----
  const float l_tot = half_swap_sum(w.l);
  if (q_row < n && qb_exists && !(kDebugModes && p.debug_mode == 3)) {
    if (p.n_slices > 1) {  // leave the partial result of this slice to the merge kernel
      const int64_t prow = ((int64_t)bh * p.n_slices + slice) * n + q_row;
      float* orow = p.part_o + prow * D;
#pragma unroll
      for (int t = 0; t < D / 32; ++t)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          typedef float f32x4 __attribute__((ext_vector_type(4)));
          f32x4 ov;
#pragma unroll
          for (int r = 0; r < 4; ++r) ov[r] = w.o[t][4 * g + r];
          __builtin_nontemporal_store(ov, reinterpret_cast<f32x4*>(orow + 32 * t + 8 * g + 4 * h));
        }
      if (h == 0) {
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        f32x2 ml = {w.m, l_tot};
        __builtin_nontemporal_store(ml, reinterpret_cast<f32x2*>(p.part_ml + prow * 2));
      }
    } else {
      const float inv = 1.0f / l_tot;
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
  if (!persistent) return;
  }  // next work item
}

__global__ void reset_queue_kernel(uint32_t* queue) {
  if (threadIdx.x < kXcds) queue[threadIdx.x] = 0u;
}

// Merge of the per-slice partial results of a row:  M = max_s m_s,  w_s = 2^(m_s - M),
//   O = sum_s w_s Num_s / sum_s w_s l_s.   A slice that saw nothing has m_s = -inf, l_s = 0.
// One thread owns 4 value columns of one row; 32 (D = 128) or 16 (D = 64) threads per row.
template <int D>
__global__ void __launch_bounds__(256) merge_kernel(AttnParams p) {
  constexpr int TPR = D / 4;
  const int64_t row = (int64_t)blockIdx.x * (256 / TPR) + threadIdx.x / TPR;  // flat (bh, token)
  if (row >= (int64_t)p.bh * p.n) return;
  const int c4 = threadIdx.x % TPR;
  const int bh = (int)(row / p.n), tok = (int)(row % p.n);
  const int64_t prow0 = (int64_t)bh * p.n_slices * p.n + tok;
  float M = -INFINITY;
  for (int s = 0; s < p.n_slices; ++s) M = fmaxf(M, p.part_ml[(prow0 + (int64_t)s * p.n) * 2]);
  float L = 0.f, acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < p.n_slices; ++s) {
    const int64_t pr = prow0 + (int64_t)s * p.n;
    const float ws = __builtin_amdgcn_exp2f(p.part_ml[pr * 2] - M);
    L += ws * p.part_ml[pr * 2 + 1];
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p.part_o + pr * D + 4 * c4));
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[r] += ws * v[r];
  }
  const float inv = 1.0f / L;
  typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
  bf16x4 ov;
#pragma unroll
  for (int r = 0; r < 4; ++r) ov[r] = (__bf16)(acc[r] * inv);
  const int64_t head_off = (int64_t)(bh / p.H) * p.stride_b + (int64_t)(bh % p.H) * p.stride_h;
  *reinterpret_cast<bf16x4*>(p.o + head_off + (int64_t)tok * p.stride_n + 4 * c4) = ov;
  if (p.lse && c4 == 0) p.lse[row] = (M + __builtin_amdgcn_logf(L)) * kLn2;
}

template <int D, bool SPARSE, bool MULTI>
hipError_t launch(const AttnParams& p, int grid, hipStream_t stream) {
  hipLaunchKernelGGL((attn_kernel<D, SPARSE, MULTI>), dim3(grid), dim3(kWaves * 64), 0, stream, p);
  return hipGetLastError();
}

}  // namespace

hipError_t pasa_launch_attn(AttnParams p, bool sparse, int d, hipStream_t stream) {
  p.c = p.scale * kLog2e;
  p.debug_mode = 0;
#ifdef PASA_DEBUG_MODES
  if (const char* e = getenv("PASA_DEBUG_MODE")) p.debug_mode = atoi(e);
#endif
  p.q_tiles = (p.n + 127) / 128;  // 128 query rows per workgroup
  p.q_tiles_per_xcd = (p.q_tiles + kXcds - 1) / kXcds;
  if (!sparse) p.n_slices = 1;
  int grid = p.bh * kXcds * p.q_tiles_per_xcd;
  if (p.n_slices > 1) {  // persistent: two workgroups per CU (64 KB of LDS each), work queues per XCD
    p.items_per_xcd = p.bh * (p.n_slices / kXcds) * p.q_tiles;
    grid = 2 * 256;
    hipLaunchKernelGGL(reset_queue_kernel, dim3(1), dim3(64), 0, stream, p.queue);
  }
  hipError_t rc = hipErrorInvalidValue;
  const bool multi = sparse && p.group > 0 && p.group < 32;
  if (sparse && d == 128) rc = multi ? launch<128, true, true>(p, grid, stream) : launch<128, true, false>(p, grid, stream);
  else if (sparse && d == 64) rc = multi ? launch<64, true, true>(p, grid, stream) : launch<64, true, false>(p, grid, stream);
  else if (d == 128) rc = launch<128, false, false>(p, grid, stream);
  else if (d == 64) rc = launch<64, false, false>(p, grid, stream);
  if (rc != hipSuccess || p.n_slices == 1) return rc;
  const int64_t rows = (int64_t)p.bh * p.n;
  if (d == 128) {
    hipLaunchKernelGGL(merge_kernel<128>, dim3((unsigned)((rows + 7) / 8)), dim3(256), 0, stream, p);
  } else {
    hipLaunchKernelGGL(merge_kernel<64>, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, stream, p);
  }
  return hipGetLastError();
}
