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
// TWO ADJACENT query blocks of 64 tokens (waves 0,1 and waves 2,3).  In the second case the key
// blocks that both query blocks selected are handled first, every tile serving all four waves
// (adjacent query blocks of a video select heavily overlapping key blocks, so this cuts the K/V
// traffic per query block); then the blocks that only one of the two selected, each wave pair on
// a tile of its own at the same time; then the approximation of the unselected blocks.  An online
// softmax does not care in which order the keys arrive.
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
// through a ring of four 16 KB LDS buffers by direct global->LDS loads: the exact passes consume a
// (K, V) pair per step while the next pair lands in the other two buffers, the approximation pass
// one tile per step with the requests three tiles ahead; one workgroup barrier per step (two in
// the pass that works on two different tiles at once).  The MFMA sequences with their operand
// fetches, and the softmax arithmetic in their shadow, are the generated instruction streams of
// pasa_mfma_pipes.hpp.
#include "pasa_device.hpp"
#include "pasa_kernels.hpp"
#include "pasa_mfma_pipes.hpp"

namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr int kXcds = 8;    // accelerator complex dies of an MI355X, each with its own L2
constexpr int kWaves = 4;   // waves per workgroup
constexpr int kRing = 4;    // LDS tile buffers
constexpr int kNoBlock = 0x7fffffff;

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
// updates the running maximum and normaliser and leaves the P^T fragments.  Only the tile rows
// [first, end) count as keys (a tile that would reach beyond the last token is fetched shifted back, so
// its leading rows belong to the tile before it; see the tile requests in the kernel).  The window
// may be empty.
template <int D>
PASA_DEVICE void exact_tile_softmax(f32x16& s0, f32x16& s1, WaveState<D>& w, float c, int first, int end, int lane,
                                    bf16x8 (&pf)[4]) {
  if (first > 0 || end < 64) {
    const int f = first - 4 * (lane >> 5), e = end - 4 * (lane >> 5);  // key = 8g + r + 4h is valid iff f <= 8g + r < e
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int key = mfma_row(r, 0);
      if (key < f || key >= e) s0[r] = -INFINITY;
      if (key + 32 < f || key + 32 >= e) s1[r] = -INFINITY;
    }
  }
  float mx = fmaxf(s0[0], s1[0]);
#pragma unroll
  for (int r = 1; r < 16; ++r) mx = max3(mx, s0[r], s1[r]);
  mx = half_swap_max(mx) * c;
  if (__builtin_amdgcn_ballot_w64(mx > w.m)) rescale<D>(w, fmaxf(w.m, mx));
  const float neg = w.m == -INFINITY ? 0.f : -w.m;  // nothing seen yet and nothing valid here: P = exp2(-inf) = 0
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
// side (which 16-byte chunk of its row a lane fetches).  Wave w issues instructions w, w+4, ... of a
// tile; a lane's rows in them are a multiple of 16 apart, so its swizzle is the same in all of them.
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
  static constexpr int STEP = kWaves * RPI;         // a lane's rows in consecutive instructions are this far apart
  static_assert(STEP % 16 == 0, "a lane's swizzle must be the same in all of its instructions");

  int row0;       // the lane's row in the wave's first instruction
  uint32_t coff;  // byte offset of the lane's (swizzled) chunk inside its row
  PASA_DEVICE void init(int wave, int lane) {
    row0 = wave * RPI + lane / CPR;
    coff = (uint32_t)(((lane % CPR) ^ swz<D>(row0)) << 4);
  }
  // Per-lane byte offsets of the wave's NI loads of a tile, relative to the tile's first row.  Rows are
  // clamped to n_rows - 1: a no-op for a matrix of at least 64 rows (tiles are requested such that
  // they lie inside it), and for a shorter one the rows that do not exist re-read the last row.
  PASA_DEVICE void offsets(uint32_t row_bytes, int n_rows, uint32_t (&x)[NI]) const {
#pragma unroll
    for (int i = 0; i < NI; ++i) x[i] = (uint32_t)min(row0 + STEP * i, n_rows - 1) * row_bytes + coff;
  }
  // Requests this wave's share of the tile whose first row is at `base` (wave-uniform).
  // lds_wave: LDS address of the slot plus wave*1024.
  PASA_DEVICE static void request(const void* base, const uint32_t (&x)[NI], uint32_t lds_wave) {
#pragma unroll
    for (int i = 0; i < NI; ++i) dma_1k(base, x[i], lds_wave + (uint32_t)(i * kWaves * 1024));
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

// ---- walking a selection bitmap ------------------------------------------------------------------
// Yields, in ascending order, the key blocks whose bit is set in a combination of (up to) two bitmap
// rows, within a range of 32-bit words.  MODE 0: blocks in both rows; 1: in row a only; 2: in row b
// only; 3: row a as it is.  The rows are held in registers, a window of 64 words (2048 key blocks) at a
// time: lane i keeps word (window + i), a ballot says which words are not empty, and the next block is
// two find-first-set steps and a lane read away -- no memory access and no loop over empty words on the
// way from one block to the next.  (With the words fetched from memory as they were needed, the scalar
// load's latency sat in front of every tile step that moved on to a new word.)  The yielded values are
// wave-uniform.
template <int MODE>
struct BitWalk {
  const_u32* ra;
  const_u32* rb;
  int w_lo, w_end;  // word range of the walk
  int win;          // first word of the window in registers
  uint32_t words;   // per lane: the combined word (win + lane), zero outside the range
  uint64_t nz;      // lanes of the window whose word still has to be visited
  uint32_t cur;     // bits of the current word that are still to be yielded
  int wi;           // index of the current word
  PASA_DEVICE void load_window(int lane) {
    const int i = win + lane;
    uint32_t a = 0u, b = 0u;
    if (i >= w_lo && i < w_end) {
      a = ra[i];
      if constexpr (MODE != 3) b = rb[i];
    }
    combine(a, b);
  }
  PASA_DEVICE void combine(uint32_t a, uint32_t b) {
    words = MODE == 3 ? a : MODE == 0 ? (a & b) : MODE == 1 ? (a & ~b) : (b & ~a);
    nz = __builtin_amdgcn_ballot_w64(words != 0u);
  }
  // first_a, first_b: word (w0 + lane) of the two rows, zero at and beyond w1 (fetched once by the caller for all
  // the walks over the same rows)
  PASA_DEVICE void init(const_u32* a, const_u32* b, int w0, int w1, uint32_t first_a, uint32_t first_b) {
    ra = a; rb = b; w_lo = w0; w_end = w1;
    win = w0; cur = 0u; wi = w0;
    combine(first_a, first_b);
  }
  PASA_DEVICE int next(int lane) {  // kNoBlock when exhausted (and on every later call)
    if (cur == 0u) {
      while (nz == 0ull) {
        if (win + 64 >= w_end) return kNoBlock;
        win += 64;
        load_window(lane);
      }
      const int l = __builtin_ctzll(nz);
      nz &= nz - 1ull;
      wi = win + l;
      cur = (uint32_t)__builtin_amdgcn_readlane((int)words, l);
    }
    const int j = __builtin_ctz(cur);
    cur &= cur - 1u;
    return 32 * wi + j;
  }
};

// Kernel variants.  MODE 0: dense (every tile); 1: sparse, one 128-token query block per workgroup;
// 2: sparse, two adjacent 64-token query blocks per workgroup.  MULTI: the group has fewer than 32
// blocks, so a chunk of 32 blocks intersects several groups and the per-block weights of a chunk have
// to be kept until all of its group matrices have passed.  SLICED: key-range slicing (persistent
// workgroups, partial results).
template <int D, int MODE, bool MULTI, bool SLICED>
__global__ void __launch_bounds__(kWaves * 64, 2) attn_kernel(AttnParams p) {
  constexpr bool SPARSE = MODE != 0;
  constexpr int TILE_BYTES = 64 * 2 * D;
  constexpr int NI = TileDma<D>::NI;
  constexpr int HPARTS = D / 64;  // 64-row tiles per group matrix
  __shared__ __attribute__((aligned(1024))) char ring[kRing * TILE_BYTES];

  __shared__ int s_item, s_queue;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ql = lane & 31, h = lane >> 5;
  const uint32_t ring_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)ring;
  LaneOffsets<D> lo;
  lo.init(lane);
  TileDma<D> dma;
  dma.init(wave, lane);
  const uint32_t row_bytes = (uint32_t)(p.stride_n * 2);
  uint32_t x_kv[NI];  // lane offsets of the loads of a whole K or V tile
  dma.offsets(row_bytes, p.n, x_kv);
  const uint32_t ring_wave = ring_base + (uint32_t)(wave * 1024);
  auto slot = [&](int i) -> uint32_t { return ring_base + (uint32_t)((i & (kRing - 1)) * TILE_BYTES); };
  auto slot_wave = [&](int i) -> uint32_t { return ring_wave + (uint32_t)((i & (kRing - 1)) * TILE_BYTES); };
  int xcd = blockIdx.x % kXcds;
  if constexpr (SLICED) {  // ask the hardware which XCD this workgroup really runs on
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
  if constexpr (SLICED) {
    // An item of this XCD's queue; once that is empty, of the next non-empty one, so that every item is computed
    // whichever XCDs the workgroups of the launch run on (fewer than eight, a masked or partitioned device).
    if (tid == 0) {
      int got = -1, from = xcd;
      for (int t = 0; t < kXcds && got < 0; ++t) {
        from = (xcd + t) % kXcds;
        const int x = (int)atomicAdd(p.queue + from, 1u);
        if (x < p.items_per_xcd) got = x;
      }
      s_item = got;
      s_queue = from;
    }
    __syncthreads();
    const int item = __builtin_amdgcn_readfirstlane(s_item);
    const int from = __builtin_amdgcn_readfirstlane(s_queue);
    __syncthreads();  // everyone has read the item before it can be written again
    if (item < 0) return;  // all queues empty: every wave of the workgroup leaves here
    const int rounds = p.n_slices / kXcds;
    const int hr = item / p.q_tiles;
    slice = (hr % rounds) * kXcds + from;
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
  // The queries are fetched together with the first tile pair (below): the two latencies overlap.
  auto load_q = [&]() {
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      uint4 raw = {0u, 0u, 0u, 0u};
      if (q_row < n) raw = *reinterpret_cast<const uint4*>(qb + (int64_t)q_row * p.stride_n + 16 * s + 8 * h);
      w.qf[s] = __builtin_bit_cast(bf16x8, raw);
    }
  };
  // Have the query loads land here.  Otherwise the compiler, which cannot see the tile loads written in
  // assembly, waits for "all loads" at the first use of Q inside the tile loops, in every iteration, and
  // so also for the tiles that were requested just before -- the prefetch would never overlap the math.
  // (Its wait covers the tile loads requested between the query loads and this point as well; the first
  // step of the tile loop needs those anyway.)
  auto settle_q = [&]() {
#pragma unroll
    for (int s = 0; s < D / 16; ++s) asm volatile("" : "+v"(w.qf[s]));
  };
#pragma unroll
  for (int t = 0; t < D / 32; ++t) w.o[t] = f32x16{0};
  w.m = -INFINITY;
  w.l = 0.f;

  // ---- the selection bitmaps of the workgroup ----
  // MODE 2: waves 0, 1 work for query block 2 qt (row a of the bitmap), waves 2, 3 for block 2 qt + 1
  // (row b).  If the last query tile has no second block, row b := row a; waves 2, 3 then repeat the
  // walk of the first block with all-zero queries (their rows lie beyond n and are never stored).
  const bool second = MODE == 2 && (wave >> 1);
  const int n_dense_tiles = (n + 63) / 64;
  const bool approx_on = SPARSE && p.group > 0;
  const uint16_t* const st = approx_on ? p.st + (int64_t)bh * p.n_chunks * 64 * D : nullptr;
  const uint16_t* const hg = approx_on ? p.hg + (int64_t)bh * p.n_groups * D * D : nullptr;
  // chunk (= bitmap word) range of this workgroup's key slice
  // (wave-uniform; the divisions run on the vector unit, so the results are moved to scalar registers explicitly)
  const int c_lo = SPARSE ? __builtin_amdgcn_readfirstlane((int)((int64_t)slice * p.n_chunks / p.n_slices)) : 0;
  const int c_hi = SPARSE ? __builtin_amdgcn_readfirstlane((int)((int64_t)(slice + 1) * p.n_chunks / p.n_slices)) : 0;
  const int qb_a = MODE == 2 ? 2 * qt : qt;
  const_u32* const mask_a = SPARSE ? (const_u32*)(p.mask + ((int64_t)bh * p.nb + qb_a) * p.mask_words) : nullptr;
  const_u32* const mask_b = (MODE == 2 && qb_a + 1 < p.nb) ? mask_a + p.mask_words : mask_a;
  const_u32* const mask_row = second ? mask_b : mask_a;  // this wave's own row
  // the first 64 words of the two rows, lane i word c_lo + i: every walk below starts from them
  uint32_t first_a = 0u, first_b = 0u;
  if constexpr (SPARSE) {
    if (c_lo + lane < c_hi) {
      first_a = mask_a[c_lo + lane];
      first_b = mask_b[c_lo + lane];
    }
  }

  // Tile requests.  The tile for key rows [r0, r0 + 64) is fetched from row tile_row(r0) on: shifted
  // back where it would reach beyond the last token, so that all 64 rows exist (r0 may even lie beyond
  // n: the second tile of the last 128-token block).  The consumer ignores the rows before r0.  Every
  // request has the same form, either here or in the shadow of MFMAs (the *_dma sequences).
  auto tile_row = [&](int r0) -> int { return max(min(r0, n - 64), 0); };
  auto tile_ptr = [&](const uint16_t* base, int r0) -> const char* {
    return reinterpret_cast<const char*>(base) + (uint32_t)tile_row(r0) * row_bytes;
  };
  auto request = [&](const uint16_t* base, int r0, int sl) { TileDma<D>::request(tile_ptr(base, r0), x_kv, slot_wave(sl)); };


  // ---------------- exact attention, part 1: tiles that all four waves need ----------------
  // (every tile of the dense path; the blocks of a 128-token query block; with two 64-token query
  // blocks the key blocks that BOTH selected).  One barrier per (K tile, V tile) pair; while a pair is
  // consumed the next pair is on its way into the other two ring slots, requested in the shadow of
  // the first MFMAs.  The order in which key blocks are visited does not matter to an online softmax.
  {
    BitWalk<MODE == 2 ? 0 : 3> walk;
    int blk = kNoBlock, sub = 0, dense_next = 0;
    if constexpr (SPARSE) {
      walk.init(mask_a, mask_b, c_lo, c_hi, first_a, first_b);
      blk = walk.next(lane);
    }
    auto plan = [&]() -> int {  // first row of the next tile, or -1
      if constexpr (MODE == 0) {
        const int t = dense_next++;
        return t < n_dense_tiles ? t * 64 : -1;
      } else if constexpr (MODE == 1) {  // two tiles per 128-token block
        if (blk == kNoBlock) return -1;
        const int r0 = blk * 128 + sub * 64;
        if (++sub == 2) { sub = 0; blk = walk.next(lane); }
        return r0;
      } else {
        if (blk == kNoBlock) return -1;
        const int r0 = blk * 64;
        blk = walk.next(lane);
        return r0;
      }
    };
    int r_cur = plan();
    load_q();
    if (r_cur >= 0) { request(kb, r_cur, 0); request(vb, r_cur, 1); }
    settle_q();
    int pair = 0;
    // Tiles whose 64 rows are all keys of the tile: one instruction stream per tile.  (Tiles come in ascending
    // order, so a tile that reaches beyond the last token can only be among the last ones.)
#pragma unroll 1
    while (r_cur >= 0 && r_cur + 64 <= n) {
      ring_barrier<NI>(0);  // the pair has landed; every wave is done with the previous pair
      const int r_nxt = plan();
      // the next pair is requested into the other two slots (after the last pair: once more the same, unused)
      const int r_req = r_nxt >= 0 ? r_nxt : r_cur;
      const uint32_t k_tile = slot(2 * pair), v_tile = slot(2 * pair + 1);
      pipes::fused_step(k_tile + lo.k, v_tile + lo.v[0], v_tile + lo.v[1], w.qf, w.o, w.m, w.l, p.c, tile_ptr(kb, r_req),
                        tile_ptr(vb, r_req), x_kv, slot_wave(2 * pair + 2), slot_wave(2 * pair + 3));
      r_cur = r_nxt;
      ++pair;
    }
    // The last tile(s), shifted back to end at the last token: their leading rows are not keys of the tile.
#pragma unroll 1
    while (r_cur >= 0) {
      ring_barrier<NI>(0);
      const int r_nxt = plan();
      const int r_req = r_nxt >= 0 ? r_nxt : r_cur;
      const uint32_t k_tile = slot(2 * pair), v_tile = slot(2 * pair + 1);
      f32x16 s0, s1;
      bf16x8 pf[4];  // P^T of the tile
      pipes::rows_x_q_dma(k_tile + lo.k, w.qf, s0, s1, tile_ptr(kb, r_req), tile_ptr(vb, r_req), x_kv,
                          slot_wave(2 * pair + 2), slot_wave(2 * pair + 3));
      exact_tile_softmax<D>(s0, s1, w, p.c, r_cur - tile_row(r_cur), n - tile_row(r_cur), lane, pf);
      pipes::cols_x_p64(v_tile + lo.v[0], v_tile + lo.v[1], pf, w.o);
      r_cur = r_nxt;
      ++pair;
    }
  }

  // ---------------- exact attention, part 2: key blocks that only one of the two query blocks selected ----------------
  // Step i handles the i-th such block of the first query block (waves 0, 1; K in slot 0, V in slot 1)
  // and the i-th of the second (waves 2, 3; slots 2, 3) at the same time, so that no wave idles.  A
  // buffer cannot be refilled while it is in use, hence two barriers per step: the V tiles of a step
  // are requested after the first and land during the logits and the softmax, the K tiles of the next
  // step are requested after the second and land during P V.
  if constexpr (MODE == 2) {
    BitWalk<1> only_a;
    BitWalk<2> only_b;
    only_a.init(mask_a, mask_b, c_lo, c_hi, first_a, first_b);
    only_b.init(mask_a, mask_b, c_lo, c_hi, first_a, first_b);
    int a_blk = only_a.next(lane), b_blk = only_b.next(lane);
    if (a_blk != kNoBlock || b_blk != kNoBlock) {
      ring_barrier<NI>(0);  // every wave is done with the ring
      request(kb, (a_blk != kNoBlock ? a_blk : b_blk) * 64, 0);
      request(kb, (b_blk != kNoBlock ? b_blk : a_blk) * 64, 2);
      // Steps in which both query blocks have a block of their own whose 64 rows are all keys: logits and
      // softmax as one instruction stream.  (Blocks come in ascending order, so the ragged last block and the
      // steps in which one list has run out can only be the last ones.)
      auto whole = [&](int blk) -> bool { return blk != kNoBlock && blk * 64 + 64 <= n; };
      const uint32_t k_mine = slot(second ? 2 : 0), v_mine = slot(second ? 3 : 1);
#pragma unroll 1
      while (whole(a_blk) && whole(b_blk)) {
        ring_barrier<NI>(0);  // the K tiles have landed; the V slots are free
        const int a_nxt = only_a.next(lane), b_nxt = only_b.next(lane);
        const int a_rq2 = a_nxt != kNoBlock ? a_nxt : b_nxt != kNoBlock ? b_nxt : a_blk;
        const int b_rq2 = b_nxt != kNoBlock ? b_nxt : a_rq2;
        bf16x8 pf[4];
        pipes::logits_softmax(k_mine + lo.k, w.qf, w.o, w.m, w.l, p.c, pf, tile_ptr(vb, a_blk * 64), tile_ptr(vb, b_blk * 64),
                              x_kv, slot_wave(1), slot_wave(3));
        ring_barrier<NI>(0);  // the V tiles have landed; the K slots are free
        pipes::cols_x_p64_dma(v_mine + lo.v[0], v_mine + lo.v[1], pf, w.o, tile_ptr(kb, a_rq2 * 64), tile_ptr(kb, b_rq2 * 64),
                              x_kv, slot_wave(0), slot_wave(2));
        a_blk = a_nxt;
        b_blk = b_nxt;
      }
#pragma unroll 1
      while (a_blk != kNoBlock || b_blk != kNoBlock) {
        ring_barrier<NI>(0);  // the K tiles have landed; the V slots are free
        // With key-range slicing one of the two query blocks can run out of blocks before the other.
        // Its waves then go through the motions on the other block's tiles with an empty key window
        // (all weights zero), and the missing tile requests repeat the other block's: one code path.
        const bool have_a = a_blk != kNoBlock, have_b = b_blk != kNoBlock;
        const int my_blk = second ? b_blk : a_blk;
        const bool read_b = second ? have_b : !have_a;  // whose slots this wave reads
        const uint32_t k_tile = slot(read_b ? 2 : 0), v_tile = slot(read_b ? 3 : 1);
        const int a_req = have_a ? a_blk : b_blk, b_req = have_b ? b_blk : a_blk;
        const int a_nxt = have_a ? only_a.next(lane) : kNoBlock;
        const int b_nxt = have_b ? only_b.next(lane) : kNoBlock;
        const int a_rq2 = a_nxt != kNoBlock ? a_nxt : b_nxt != kNoBlock ? b_nxt : a_req;
        const int b_rq2 = b_nxt != kNoBlock ? b_nxt : a_rq2;
        const int t_row = my_blk != kNoBlock ? tile_row(my_blk * 64) : 0;
        const int first = my_blk != kNoBlock ? my_blk * 64 - t_row : 64, end = my_blk != kNoBlock ? n - t_row : 64;
        f32x16 s0, s1;
        bf16x8 pf[4];
        pipes::rows_x_q_dma(k_tile + lo.k, w.qf, s0, s1, tile_ptr(vb, a_req * 64), tile_ptr(vb, b_req * 64), x_kv,
                            slot_wave(1), slot_wave(3));
        exact_tile_softmax<D>(s0, s1, w, p.c, first, end, lane, pf);
        ring_barrier<NI>(0);  // the V tiles have landed; the K slots are free
        pipes::cols_x_p64_dma(v_tile + lo.v[0], v_tile + lo.v[1], pf, w.o, tile_ptr(kb, a_rq2 * 64),
                              tile_ptr(kb, b_rq2 * 64), x_kv, slot_wave(0), slot_wave(2));
        a_blk = a_nxt;
        b_blk = b_nxt;
      }
    }
  }

  // ---------------- grouped approximation of the unselected blocks ----------------
  // Per chunk of 32 key blocks: its statistics tile, then for every group it intersects the HPARTS
  // tiles of the group matrix.  The tiles stream through the ring three ahead of their use, one
  // barrier per tile.
  uint32_t x_ws[NI];  // lane offsets of the loads of a workspace tile (rows of D elements)
  dma.offsets(2 * D, 64, x_ws);
  int c_slow = c_lo;  // first chunk left to the general loop below
  // Groups of whole chunks (a multiple of 32 blocks), chunks whose 32 blocks all exist and are full: a fixed
  // sequence of tiles (the statistics of a group's chunks, then the HPARTS tiles of its matrix), each handled by
  // one instruction stream that also requests the tile three further down the stream.  (The last chunk of the
  // sequence may be short; it takes the general loop.)
  if constexpr (SPARSE && !MULTI) {
    const int c_fast = approx_on ? min(c_hi, p.n_chunks - 1) : 0;
    if (c_lo < c_fast) {
      // chunks per group (a group size that is not a multiple of 32 is the single group that spans all blocks)
      const int cpg = (p.group & 31) == 0 ? p.group >> 5 : p.n_chunks;
      // the tile that is requested next: kind 0 = statistics of chunk rq_c, kind 1.. = that part of its group's matrix
      int rq_c = c_lo, rq_kind = 0, rq_g = __builtin_amdgcn_readfirstlane(c_lo / cpg);  // (the division runs on the vector unit)
      int rq_left = cpg - (c_lo - rq_g * cpg);  // chunks from rq_c to the end of its group
      auto rq_ptr = [&]() -> const char* {
        const uint64_t a = (uint64_t)(rq_kind == 0 ? st + (int64_t)rq_c * 64 * D : hg + ((int64_t)rq_g * D + 64 * (rq_kind - 1)) * D);
        // wave-uniform by construction; said explicitly because the instruction streams take it in scalar registers
        // (the intrinsic returns a signed int: back to unsigned before widening, or the low half would sign-extend)
        const uint32_t a_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)a);
        const uint32_t a_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(a >> 32));
        return reinterpret_cast<const char*>((uint64_t)a_lo | ((uint64_t)a_hi << 32));
      };
      // The group matrix follows the statistics of the LAST chunk of its group (and of the last chunk of this loop,
      // should the group go on beyond it): the first-order term is linear in the group weight, so the weights of a
      // group's chunks are summed and the matrix is applied once.
      // (after the last tile: the last chunk's statistics over and over, into slots that nobody reads any more)
      bool rq_done = false;
      auto rq_advance = [&]() {
        if (rq_done) return;
        const bool last_chunk = rq_c + 1 >= c_fast;
        if (rq_kind == 0) {
          if (rq_left == 1 || last_chunk) {
            rq_kind = 1;  // the group's matrix follows
          } else {        // the next chunk belongs to the same group
            ++rq_c;
            --rq_left;
          }
        } else if (rq_kind < HPARTS) {
          ++rq_kind;
        } else {
          rq_kind = 0;
          if (last_chunk) {
            rq_done = true;
          } else {
            ++rq_c;
            if (--rq_left == 0) { ++rq_g; rq_left = cpg; }
          }
        }
      };
      ring_barrier<NI>(0);  // every wave is done with the ring
      for (int i = 0; i < 3; ++i) {
        TileDma<D>::request(rq_ptr(), x_ws, slot_wave(i));
        rq_advance();
      }
      const float bf = (float)p.block;
      const uint32_t sh = (uint32_t)(4 * h);
      int t = 0;  // tiles consumed so far; tile t is in ring slot t & 3
      float A_group = 0.f;                       // sum of the a_j of the group's chunks so far: the weight of its first-order term
      int left = cpg - (c_lo - (c_lo / cpg) * cpg);  // chunks from `chunk` to the end of its group
#pragma unroll 1
      for (int chunk = c_lo; chunk < c_fast; ++chunk) {
        float A;
        ring_barrier<NI>(2);
        pipes::stats_step(slot(t) + lo.k, slot(t) + lo.v[0], slot(t) + lo.v[1], w.qf, w.o, w.m, w.l, p.c, ~mask_row[chunk], sh, bf,
                          A, rq_ptr(), x_ws, slot_wave(t + 3));
        rq_advance();
        ++t;
        A_group += A;
        if (--left != 0 && chunk + 1 < c_fast) continue;
        left = cpg;
        ring_barrier<NI>(2);
        pipes::first_order_step0(slot(t) + lo.k, w.qf, w.o, A_group, rq_ptr(), x_ws, slot_wave(t + 3));
        rq_advance();
        ++t;
        if constexpr (D == 128) {
          ring_barrier<NI>(2);
          pipes::first_order_step1(slot(t) + lo.k, w.qf, w.o, A_group, rq_ptr(), x_ws, slot_wave(t + 3));
          rq_advance();
          ++t;
        }
        A_group = 0.f;
      }
      c_slow = c_fast;
    }
  }
  // General loop: the consumer learns what a tile is from a descriptor:
  //   bits 0-2 kind;  bits 3-15 chunk (at most 8192 chunks);  bits 16-31 group (at most 65535 groups; the host checks both)
  if (approx_on && c_slow < c_hi) {
    enum : uint32_t { kEnd = 0, kStats = 3, kHPart = 4 };
    ring_barrier<NI>(0);  // every wave is done with the ring, and no request is in flight
    int issued = 0;       // tiles requested so far; tile i goes to ring slot i & 3
    int it = 0;           // tiles consumed so far
    int p_chunk = c_slow, p_group = 0, p_part = -1;  // p_part == -1: statistics tile next
    auto produce = [&]() -> uint32_t {
      if (p_chunk >= c_hi) return kEnd;
      uint32_t desc;
      const uint16_t* src;
      if (p_part < 0) {
        src = st + (int64_t)p_chunk * 64 * D;
        desc = kStats | ((uint32_t)p_chunk << 3);
        p_group = (32 * p_chunk) / p.group;
        p_part = 0;
      } else {
        src = hg + ((int64_t)p_group * D + 64 * p_part) * D;
        desc = kHPart | ((uint32_t)p_chunk << 3) | ((uint32_t)p_group << 16);
        if (++p_part == HPARTS) {
          p_part = 0;
          if (++p_group > (min(32 * p_chunk + 32, p.nb) - 1) / p.group) { ++p_chunk; p_part = -1; }
        }
      }
      TileDma<D>::request(src, x_ws, slot_wave(issued));
      ++issued;
      return desc;
    };
    uint32_t d0 = produce(), d1 = produce(), d2 = kEnd;  // tiles requested but not yet consumed, in order
    // Moves on to the next tile of the stream: waits for it, meets the other waves (after which the
    // slots of all earlier tiles are free) and tops the ring up to three tiles ahead.  Returns the
    // descriptor of the tile to consume (slot(it)).
    auto next_tile = [&]() -> uint32_t {
      const uint32_t cur = d0;
      ring_barrier<NI>((d1 != kEnd ? 1 : 0) + (d2 != kEnd ? 1 : 0));
      d0 = d1;
      d1 = d2;
      d2 = kEnd;
      if (d0 == kEnd) d0 = produce();
      if (d1 == kEnd && d0 != kEnd) d1 = produce();
      if (d2 == kEnd && d1 != kEnd) d2 = produce();
      return cur;
    };
#pragma unroll 1
    while (d0 != kEnd) {
      f32x16 a;  // a_j of the chunk
      const uint32_t cur = next_tile();
      const int chunk = (int)((cur >> 3) & 8191u);
      approx_chunk_zeroth<D>(slot(it), lo, w, p.c, mask_row[chunk], chunk, p.nb, p.block, p.tail, lane, a);
      ++it;
      float A = 0.f;
      if constexpr (!MULTI) {  // the whole chunk belongs to one group
#pragma unroll
        for (int r = 0; r < 16; ++r) A += a[r];
        A = half_swap_sum(A);
      }
#pragma unroll 1
      while ((d0 & 7u) == kHPart) {
        if constexpr (MULTI) {
          const int g = (int)(d0 >> 16);
          A = 0.f;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = 32 * chunk + mfma_row(r, h);
            A += (j / p.group == g) ? a[r] : 0.f;
          }
          A = half_swap_sum(A);
        }
        next_tile();
        first_order_part<D, 0>(slot(it), lo, w, A);
        ++it;
        if constexpr (D == 128) {
          next_tile();
          first_order_part<D, 1>(slot(it), lo, w, A);
          ++it;
        }
      }
    }
  }

  // ---- epilogue ----
  // The last steps of the tile loops repeat a request that nobody consumes: let those loads land
  // before this workgroup's LDS can be handed to another one.
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  const float l_tot = half_swap_sum(w.l);
  if (q_row < n) {
    if constexpr (SLICED) {  // leave the partial result of this slice to the merge kernel
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
  if constexpr (!SLICED) return;
  // the next item's first requests must not overtake the last LDS reads of slower waves
  ring_barrier<NI>(0);
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

template <int D, int MODE, bool MULTI, bool SLICED>
hipError_t launch(const AttnParams& p, int grid, hipStream_t stream) {
  hipLaunchKernelGGL((attn_kernel<D, MODE, MULTI, SLICED>), dim3(grid), dim3(kWaves * 64), 0, stream, p);
  return hipGetLastError();
}

template <int D>
hipError_t launch_d(const AttnParams& p, bool sparse, int grid, hipStream_t stream) {
  if (!sparse) return launch<D, 0, false, false>(p, grid, stream);
  const bool multi = p.group > 0 && p.group < 32, sliced = p.n_slices > 1;
  if (p.block == 128) {
    if (sliced) return multi ? launch<D, 1, true, true>(p, grid, stream) : launch<D, 1, false, true>(p, grid, stream);
    return multi ? launch<D, 1, true, false>(p, grid, stream) : launch<D, 1, false, false>(p, grid, stream);
  }
  if (sliced) return multi ? launch<D, 2, true, true>(p, grid, stream) : launch<D, 2, false, true>(p, grid, stream);
  return multi ? launch<D, 2, true, false>(p, grid, stream) : launch<D, 2, false, false>(p, grid, stream);
}

}  // namespace

hipError_t pasa_launch_attn(AttnParams p, bool sparse, int d, hipStream_t stream) {
  p.c = p.scale * kLog2e;
  p.q_tiles = (p.n + 127) / 128;  // 128 query rows per workgroup
  p.q_tiles_per_xcd = (p.q_tiles + kXcds - 1) / kXcds;
  if (!sparse) p.n_slices = 1;
  int grid = p.bh * kXcds * p.q_tiles_per_xcd;
  if (p.n_slices > 1) {  // persistent: two workgroups per CU (64 KB of LDS each), work queues per XCD
    p.items_per_xcd = p.bh * (p.n_slices / kXcds) * p.q_tiles;
    int dev = 0, cus = 0;  // host queries only: nothing is allocated or synchronised
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) {
      (void)hipGetLastError();
      cus = 256;
    }
    grid = 2 * cus;
    hipLaunchKernelGGL(reset_queue_kernel, dim3(1), dim3(64), 0, stream, p.queue);
  }
  const hipError_t rc = d == 128 ? launch_d<128>(p, sparse, grid, stream) : launch_d<64>(p, sparse, grid, stream);
  if (rc != hipSuccess || p.n_slices == 1) return rc;
  const int64_t rows = (int64_t)p.bh * p.n;
  if (d == 128) {
    hipLaunchKernelGGL(merge_kernel<128>, dim3((unsigned)((rows + 7) / 8)), dim3(256), 0, stream, p);
  } else {
    hipLaunchKernelGGL(merge_kernel<64>, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, stream, p);
  }
  return hipGetLastError();
}
