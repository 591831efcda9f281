// FlashAttention-style forward kernels for gfx950 (MI355X): dense attention, the
// block-sparse pass over a kept-tile list (Sec. 4.3), and the masked passes of online
// profiling over sampled query rows (Alg. 1, Sec. 4.1).
//
// One workgroup owns one query tile of one head; each of its NW wavefronts owns 32
// query rows and all BN keys of the current key tile.  Both matrix products are
// computed TRANSPOSED with v_mfma_f32_32x32x16_bf16:
//     S^T = K Q^T      (A = K tile from LDS,  B = Q^T held in registers)
//     O^T += V^T P^T   (A = V^T from LDS,     B = P^T taken from S^T's registers)
// In the 32x32 accumulator layout a lane holds ONE query column (lane % 32) and 16
// key rows, so the softmax row statistics are per-lane register reductions plus one
// exchange between lane l and lane l+32, the rescale factor is one scalar per lane,
// and the exponentiated S^T registers are, after bf16 packing, exactly the B operand
// of the second product: register pair (2kk, 2kk+1) of a 32-key block holds keys
// {16kk+4g+j} and {16kk+8+4g+j}, j<4, g = lane/32, and the V^T operand is read in
// the same key order, so P never moves between lanes or through LDS.
//
// Staging: K and V tiles go global -> registers (raw buffer loads, bounds-checked
// descriptors, loop-invariant offsets) -> LDS as straight 16-byte copies, double
// buffered, with the loads of tile j+1 in flight while tile j is computed and one
// barrier per tile.  K rows are padded by 16 bytes (conflict-free ds_read_b128 of the A
// operand with compile-time offsets).  V stays row-major too: the transposing LDS read
// of gfx950 (ds_read_b64_tr_b16) hands a lane the same channel of four consecutive
// keys, so two of them are a whole A operand of the second product and nothing is
// transposed in registers.  Operand reads run a few
// products ahead of their use (rolling window), including the first V^T operands,
// which are requested before the softmax starts.
//
// Softmax: fp32, base-2 exponentials with scale * log2 e folded into one FMA per
// element.  The exponentials are taken against the current reference maximum without
// looking at the tile's own maximum; only when a row sum shows that the reference is
// too small does the wave fall back to the classic update (tile maximum, rescale).
// P is rounded to bf16 for the second product; accumulation is fp32; the running sum
// uses the unrounded P at head dimension 128 and the rounded P at head dimension 64.
//
// Measured on MI355X:
//  * With 32 query rows per wavefront every MFMA needs a fresh 1 KB operand from LDS.  The
//    LDS reads 256 B/clk per CU (two or more wavefronts per SIMD; a lone one reaches
//    half of that) and writes 79 B/clk; operand reads and staging writes together keep
//    it busy about 55 % of the time at the speed reached here, the matrix cores 59 %.
//  * The chip is power-limited under this load: the shader clock sits near 1.7 GHz (2.4 GHz
//    nominal), and a loop of nothing but MFMAs on random operands is held there too.  A
//    variant that idles more runs at a higher clock and ends up at the same rate; what
//    pays is less work per tile (instructions, LDS and memory traffic), not fewer cycles.
//  * A lone wavefront hides only about 12 cycles of other instructions behind each
//    32-cycle MFMA; two wavefronts on a SIMD overlap one's VALU work with the other's
//    products much better, and best when each runs long homogeneous phases (products /
//    softmax) and the one issuing products has the higher wave priority.  Interleaving
//    softmax slices between the products of the same wavefront was 10 % slower.
//  * 64 query rows per wavefront (every LDS operand feeding two products) needs more than
//    the 256 registers a wavefront has at two per SIMD; with one wavefront per SIMD it
//    loses the overlap above and was 5 % slower.  A 256-row workgroup (two query tiles
//    sharing every staged tile, the two halves one phase apart) halved staging and L2
//    traffic per product and came out even: more cycles at a higher clock.
#include "svg_attn_common.h"

namespace svg {

namespace {

using namespace attn;

constexpr int kNoTile = 0x7fffffff;
// Wave priority while a wavefront issues a batch of products (0 elsewhere).  The two
// wavefronts sharing a SIMD then settle into opposite phases: the products of one run
// back to back while the other's softmax and staging instructions fill the gaps.  The first
// product of a tile ranks above the second (1 % less time than equal ranks, 1 % more with the
// ranks swapped): a wavefront that starts a tile is not held up by one that finishes one.
constexpr int kPrioFirstProduct = 2;
constexpr int kPrioSecondProduct = 1;
constexpr int kCohort = 64;   // dense: consecutive query tiles that share an XCD (and its L2) at a time
// LDS operand reads kept in flight ahead of the products: eight where the registers allow it
// (the dense and the plain sparse pass at head dimension 128; 0.3 % over four), six in the
// gathering form (0.5-0.9 % over four), four elsewhere
constexpr int prefetch_depth(int D, int NW, int MODE) {
  return D != 128 || NW != 4 ? 4 : MODE == kDense || MODE == kSparse ? 8 : MODE == kSparseGather ? 6 : 4;
}
constexpr unsigned kRsrcFlags = 0x00020000u;   // raw buffer, 32-bit data format (gfx9 encoding)

// Wavefronts per SIMD the register budget is set for.  Head dimension 128 fills 256 registers
// (two wavefronts).  At head dimension 64 the accumulators are half as large and every form fits
// 168 registers: three workgroups per CU, whose wavefronts cover each other's softmax phases
// (the longer phase at this head dimension) better than two workgroups with twice the keys per
// barrier did (4-7 % less time in the dense and sparse passes, 14 % in profiling).
constexpr int waves_per_simd(int D, int NW, int MODE) {
  return NW != 4 ? 1 : D == 64 ? 3 : 2;
}

template <int D, int NW, int BN, int MODE, int LW>
__global__ __launch_bounds__(64 * NW, waves_per_simd(D, NW, MODE)) void attn_kernel(AttnArgs a) {
  constexpr int BM = 32 * NW;            // query rows per workgroup = rows of a query tile
  constexpr int THREADS = 64 * NW;
  constexpr int CPR = D / 8;             // 16-byte pieces per row
  constexpr int KB = BN / 32;            // 32-key blocks per tile
  // kSparseExact is kSparse with the head's element mask applied inside every visited tile
  // kSparseGather is kSparse with k and v of the temporal heads left in token order: the rows of
  // a key tile are fetched from where the layout transformation would have taken them
  constexpr bool SPARSE = MODE == kSparse || MODE == kSparseExact || MODE == kSparseGather;
  constexpr bool GATHER = MODE == kSparseGather;
  static_assert(!GATHER || NW == 4, "the gathering form exists for 128-row query tiles");
  constexpr bool MASKABLE = MODE == kProfile || MODE == kSparseExact;
  constexpr int DS = D / 16;             // k-steps of the first product
  constexpr int DB = D / 32;             // 32-row blocks of O^T
  constexpr int PIECES = BN * CPR;       // 16-byte pieces of a K tile, and of a V tile
  // Staging work: every thread copies PER_THREAD pieces of K and of V, global -> registers -> LDS,
  // so all wavefronts reach the barrier with the same amount of work behind them.
  constexpr int PER_THREAD = PIECES / THREADS;
  static_assert(PIECES % THREADS == 0 && THREADS % CPR == 0, "every thread stages the same piece of whole rows");
  // K staging: row-major, rows padded by 16 bytes so that the 16 lanes served together
  // by a ds_read_b128 of the A operand (16 consecutive keys, same channel piece) fall on
  // different banks, while every operand address stays base + compile-time offset.
  constexpr int K_ROW = D * 2 + 16;
  constexpr int K_BYTES = BN * K_ROW;
  // V staging: row-major as well, not transposed.  The A operand of the second product is V^T,
  // which the transposing LDS read of gfx950 (ds_read_b64_tr_b16) delivers directly: the 16
  // lanes of a quarter wavefront read 4 rows x 16 channels (lane s: 8 bytes of row s / 4 at
  // channel 4 (s % 4)) and lane i receives channel i of the four rows.  Two such reads (rows
  // 4 g + {0..3} and 8 + 4 g + {0..3} of a 16-key step) are one operand in the key order the
  // weights are held in.  The 32-byte slots of a row are XOR-swizzled with the row's two low bits
  // (v_swizzle), which puts the four rows of a quarter wavefront, and the eight row pieces of a
  // half wavefront, on different banks; rows stay unpadded.
  constexpr int V_ROW = D * 2;
  constexpr int V_BYTES = BN * V_ROW;
  constexpr int STAGE_BYTES = K_BYTES + V_BYTES;

  __shared__ __attribute__((aligned(16))) unsigned char lds[2 * STAGE_BYTES];
  __shared__ __attribute__((aligned(16))) int key_code[MASKABLE ? 2 * BN : 4];
  // profile: per staged tile {smallest coordinate code, largest, flags}; flags bit 0: some key
  // is kept by every query, bit 1: some key is out of range, bit 2: coordinates span a wrap
  __shared__ int tile_info[MASKABLE ? 2 * 4 : 4];
  __shared__ int wg_range[4];    // profile: min / max coordinate of the workgroup's rows

  // ======================================================================================
  // Which (head, row group) is this workgroup?  Consecutive logical ids are placed on the
  // same XCD (workgroups are dealt round-robin over the 8 XCDs), so the query tiles that
  // stream the same K/V share one L2.
  // ======================================================================================
  const int xcd = blockIdx.x & 7, loc = blockIdx.x >> 3;
  int bh = 0, grp = 0, variant = 0, chunk = 0;
  if (MODE == kProfile) {
    // (head, row group) pairs are split into 8 contiguous chunks, one per XCD.  Each pair
    // has 2 n_masked + n_full units: the parts of the spatial pass, of the temporal pass (both
    // skip most key tiles) and of the unmasked pass.  Units are the outer index inside an
    // XCD's chunk, so neighbouring workgroups stream the same keys for neighbouring row
    // groups of one head.
    const int pairs = a.BH * a.nqt;
    const int pairs_per_xcd = (pairs + 7) >> 3;
    const int unit = loc / pairs_per_xcd;
    const int pair = xcd * pairs_per_xcd + (loc - unit * pairs_per_xcd);
    const int nm = a.plan.n_masked;
    if (unit >= a.plan.slots() || pair >= pairs) return;
    // the masked passes first: their workgroups are the longest ones (mask work on top of
    // about as many tiles), so they should not be the last to start
    variant = unit < nm ? 1 : unit < 2 * nm ? 2 : 0;         // 0 unmasked, 1 spatial, 2 temporal
    chunk = unit < nm ? unit : unit < 2 * nm ? unit - nm : unit - 2 * nm;    // which part of its pass
    bh = pair / a.nqt;
    grp = pair - bh * a.nqt;
  } else if (MODE == kDense) {
    // Dense: blocks of kCohort consecutive logical ids go to one XCD, consecutive blocks to
    // consecutive XCDs.  An XCD's L2 serves neighbouring query tiles of one head, and at
    // any time all XCDs work on the same one or two heads, whose K/V (61 MB per head at
    // the 120k-token shape) then stay in the memory-side cache in front of HBM; with one
    // head per XCD the dense pass runs into the HBM bandwidth (-11 % time).
    const int lid = ((loc / kCohort) * 8 + xcd) * kCohort + (loc % kCohort);
    if (lid >= a.total) return;
    bh = lid / a.nqt;
    grp = lid - bh * a.nqt;
  }
  // sparse: heavy tiles first, then an eighth of each label's sequence of tiles
  int pat = 0, cl = -1, head_cl0 = 0;
  if (SPARSE) {
    if (!sparse_slot<LW>(a.so, a.BH, a.labels, a.row_ptr[0], a.row_ptr[1], bh, grp, pat, cl, head_cl0)) return;
    bh = __builtin_amdgcn_readfirstlane(bh);
    grp = __builtin_amdgcn_readfirstlane(grp);
    pat = __builtin_amdgcn_readfirstlane(pat);
  }

  // profile: the unmasked pass needs no key codes, tile summaries or element masks (only the
  // ragged end of the sequence, handled like in the dense pass)
  const bool masked = MODE == kSparseExact || (MODE == kProfile && __builtin_amdgcn_readfirstlane(variant) != 0);

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int g = lane >> 5;       // which half of the wavefront
  const int r = lane & 31;       // query column within the wave / row of the A operand

  const size_t head = (size_t)bh * a.N;

  // ======================================================================================
  // This lane's query row, its mask window (profile), and Q^T as the B operand.
  // ======================================================================================
  int qslot = grp * BM + wave * 32 + r;     // row (profile: index into rows[])
  int qrow;
  if (MODE == kProfile) {
    // The sampled rows are dealt evenly to the row groups (rows_per_group each, so that no
    // group is left with a handful of rows and idle wavefronts); a lane without a row of
    // its own shadows the group's first row and writes nothing.
    const int in_group = wave * 32 + r;
    const int first = min(grp * a.rows_per_group, a.t - 1);
    qslot = in_group < a.rows_per_group ? grp * a.rows_per_group + in_group : a.t;
    // The temporal variant takes the sampled rows grouped by in-frame position, so that
    // a workgroup's rows share a narrow position range and most key tiles can be
    // skipped; results are still written at the row's own slot.
    int slot = qslot < a.t ? qslot : first;
    if (variant == 2) slot = a.order_t[slot];
    if (qslot < a.t) qslot = slot;
    qrow = a.rows[slot];
  } else {
    qrow = min(qslot, a.N - 1);
  }

  // profile: a key with code c is kept iff (unsigned)(c - win_lo) <= win_span or c == kCodeKeep
  int win_lo = 0;
  unsigned win_span = 0x7ffffffeu;
  if (MODE == kProfile) {
    if (tid == 0) {
      wg_range[0] = 0x7fffffff;
      wg_range[1] = -1;
    }
    __syncthreads();
    if (variant != 0 && qrow >= a.off && qrow < a.video_end) {
      const int vq = qrow - a.off;
      const int fq = vq / a.P;
      const int c = variant == 1 ? fq : vq - fq * a.P;
      const int w = variant == 1 ? a.w_s : a.w_t;
      win_lo = c - w;
      win_span = 2u * (unsigned)w;
      atomicMin(&wg_range[0], c);
      atomicMax(&wg_range[1], c);
    }
    // (a text query attends to everything under both masks, so its masked outputs equal
    // the unmasked one by definition: it adds nothing to either error, the error kernel
    // skips it, and it need not widen this workgroup's key range)
    __syncthreads();
  }

  // sparse: this head's pattern; with q and o kept in token order, the row of a temporal
  // head that this lane reads and writes is the token whose transformed position is qrow
  // (Sec. 4.2: position off + p F + f holds token off + f P + p; with the first-frame sink,
  // frame 0 leads as a block)
  // a temporal head reads the P-outer copies of k and v when the caller keeps them apart from
  // the originals (which the spatial heads read in place)
  const bool kv_copy = SPARSE && __builtin_amdgcn_readfirstlane(pat) != 0 && a.k_t != nullptr;
  const __bf16* kh = (kv_copy ? a.k_t : a.k) + head * D;
  const __bf16* vh = (kv_copy ? a.v_t : a.v) + head * D;
  int io_row = qrow;
  if (SPARSE && a.qo_token_order && pat && qrow >= a.off && qrow < a.video_end)
    io_row = a.off + (int)transformed_to_token((unsigned)(qrow - a.off), (unsigned)a.F, (unsigned)a.P, a.sink);
  if (MODE == kSparseExact && qrow >= a.off && qrow < a.video_end) {
    // element mask of the head's pattern in the order its tile list refers to: a spatial head
    // compares frames (coordinate = row / P), a temporal head in P-outer order compares in-frame
    // positions (coordinate = row / F); text queries keep the default window (everything)
    int cq = (qrow - a.off) / a.P;
    if (pat) {
      unsigned pq;
      transformed_to_token((unsigned)(qrow - a.off), (unsigned)a.F, (unsigned)a.P, a.sink, &pq);
      cq = (int)pq;
    }
    const int w = pat ? a.w_t : a.w_s;
    win_lo = cq - w;
    win_span = 2u * (unsigned)w;
  }

  bf16x8 qreg[DS];     // lane (g, r) holds Q[qrow][16 s + 8 g .. +8]
  {
    const __bf16* qp = a.q + (head + io_row) * D + g * 8;
#pragma unroll
    for (int s = 0; s < DS; ++s) qreg[s] = *reinterpret_cast<const bf16x8*>(qp + s * 16);
  }

  // ======================================================================================
  // Tile cursor: the next key tile of this workgroup, or kNoTile.
  //   dense   : 0 .. nk-1
  //   sparse  : the query tile's row of the head's CSR list
  //   profile : tiles of the key intervals that can hold a kept key for ANY row of the
  //             workgroup, ascending: text prefix | frame 0 (sink) | the window around the
  //             rows' frames (spatial) or, per frame, the window around the rows' positions
  //             (temporal) | text suffix; the unmasked pass walks its key range.  A superset
  //             is enough: the element mask is still applied inside every visited tile.
  // ======================================================================================
  const int32_t* cols = nullptr;
  int lj = 0, lend = 0;              // sparse: cursor and end in col_idx;  dense: counter and nk
  int lbeg = 0, lleft = 0;           // sparse: start of the list row, entries still to hand out
  if (SPARSE) {
    const int32_t* rp = a.row_ptr[pat];
    cols = a.col_idx[pat];
    lbeg = __builtin_amdgcn_readfirstlane(rp[grp]);
    lend = __builtin_amdgcn_readfirstlane(rp[grp + 1]);
    lj = lbeg;
    lleft = lend - lbeg;
    // The list is walked from its first entry.  Neighbouring query tiles run at the same time on
    // one XCD with key windows shifted by BM / BN tiles against each other, so each finds in L2
    // what its neighbour fetched a moment ago.  (An earlier form started all query tiles of a
    // cohort of up to 64 at one common key tile and walked the lists cyclically; with whole heads
    // dealt to the XCDs that saved a third of the traffic past L2, with the dispatch order used
    // now it cost 1-2 % time and nearly doubled that traffic: 47.9 against 27.5 GB per launch at
    // the 119k-token shape.)
  } else if (MODE == kDense) {
    lend = a.nk;
  }
  const int c_lo = MODE == kProfile ? wg_range[0] : 0, c_hi = MODE == kProfile ? wg_range[1] : -1;
  int pseg = 0, pj = 0, pjb = -1;
  auto profile_segment = [&](int sidx, int& k0, int& k1) -> bool {   // false: no more segments
    if (variant == 0) {      // unmasked pass: the key tiles of part chunk
      const int t0 = a.plan.full_bound[chunk], t1 = a.plan.full_bound[chunk + 1];
      k0 = t0 * BN;
      k1 = min(a.N, t1 * BN) - 1;
      return sidx == 0;
    }
    const int nv = variant == 1 ? 1 : a.F;
    if (sidx == 0) {            // text prefix
      k0 = 0;
      k1 = a.off - 1;
    } else if (sidx == 1) {     // first-frame sink
      k0 = a.off;
      k1 = a.sink ? a.off + a.P - 1 : a.off - 1;
    } else if (sidx < 2 + nv) {
      if (c_hi < 0) {           // every row of the workgroup is a text row: nothing to do
        k0 = 0;
        k1 = -1;
      } else if (variant == 1) {
        k0 = a.off + max(0, c_lo - a.w_s) * a.P;
        k1 = a.off + min(a.F, c_hi + a.w_s + 1) * a.P - 1;
      } else {
        const int f = sidx - 2;
        k0 = a.off + f * a.P + max(0, c_lo - a.w_t);
        k1 = a.off + f * a.P + min(a.P - 1, c_hi + a.w_t);
      }
    } else if (sidx == 2 + nv) {  // text suffix
      k0 = a.video_end;
      k1 = a.N - 1;
    } else {
      return false;
    }
    return true;
  };
  int pleft = 0x7fffffff;    // profile: tiles this workgroup may still take
  // profile: makes [pj, pjb] the next non-empty run of tiles of the pass (intervals may overlap
  // or touch; a tile is handed out once); false when the pass is exhausted
  auto profile_interval = [&]() -> bool {
    while (pj > pjb) {
      int k0, k1;
      if (!profile_segment(pseg, k0, k1)) return false;
      ++pseg;
      if (k1 < k0) continue;
      const int ja = k0 / BN, jb = k1 / BN;
      if (jb < pj) continue;
      pj = max(pj, ja);
      pjb = jb;
    }
    return true;
  };
  // The cursor works in two halves.  fetch_begin() at the top of an iteration issues the
  // loads of the next list entries; fetch_end() late in the iteration, where the staged data
  // has just been waited for anyway, turns them into the next entry and advances the
  // cursor.  The entry is needed three tiles later.  The loads are ordinary per-lane loads
  // (the opaque zero keeps the compiler from treating the address as uniform and waiting
  // for the value on the spot, which would also wait for every staging load in flight).
  int lane_zero = 0;
  asm volatile("" : "+v"(lane_zero));
  int pend0 = kNoTile;
  auto fetch_begin = [&]() {
    if (SPARSE) pend0 = lleft > 0 ? cols[lj + lane_zero] : kNoTile;
  };
  auto fetch_end = [&]() -> int {
    if (SPARSE) {
      if (lleft <= 0) return kNoTile;
      const int c = __builtin_amdgcn_readfirstlane(pend0);
      --lleft;
      ++lj;
      return c;
    }
    if (MODE == kDense) {
      const int j = lj++;
      if (j >= lend) return kNoTile;
      return j;
    }
    if (pleft <= 0) return kNoTile;     // profile
    if (!profile_interval()) return kNoTile;
    --pleft;
    return pj++;
  };
  if (MODE == kProfile && variant != 0 && a.plan.n_masked > 1) {
    // a masked pass in parts: count the tiles of the whole pass, then take the part's share
    int total = 0;
    while (profile_interval()) {
      total += pjb - pj + 1;
      pj = pjb + 1;
    }
    const int first = (int)(((long long)total * chunk) / a.plan.n_masked);
    pleft = (int)(((long long)total * (chunk + 1)) / a.plan.n_masked) - first;
    pseg = 0; pj = 0; pjb = -1;
    int skip = first;
    while (skip > 0 && profile_interval()) {
      const int n = min(skip, pjb - pj + 1);
      pj += n;
      skip -= n;
    }
  }
  auto next_tile = [&]() -> int {      // both halves at once (prologue)
    fetch_begin();
    return fetch_end();
  };

  // ======================================================================================
  // Staging of one K/V tile.
  // ======================================================================================
  u32x4 kst[PER_THREAD], vst[PER_THREAD];     // this thread's pieces of K and of V

  // The descriptor of a tile starts at the tile's first key row and covers the rows up to
  // N, so the per-thread offsets are loop invariant, no clamping arithmetic is needed, and
  // rows beyond N (ragged last tile) read as zero.  A thread stages piece tid % CPR of PER_THREAD
  // rows: rows tid / CPR + i (THREADS / CPR), so that a wavefront's load covers consecutive rows,
  // or, in the gathering form, where the rows come from anywhere, the consecutive rows
  // PER_THREAD (tid / CPR) + i, whose row numbers one load fetches.
  constexpr int ROW_STEP = GATHER ? 1 : THREADS / CPR;
  const int stage_row = (tid / CPR) * (GATHER ? PER_THREAD : 1), stage_piece = tid % CPR;
  const int stage_off = (stage_row * D + stage_piece * 8) * 2;
  // 32-byte slot s of V row n sits at slot s ^ v_swizzle(n) of the row in LDS
  auto v_swizzle = [](int n) { const int j = n & 3; return D == 128 ? (2 * j) ^ (j >> 1) : j; };
  const int k_lds_off = stage_row * K_ROW + (stage_piece << 4);
  int v_lds_off[PER_THREAD];
#pragma unroll
  for (int i = 0; i < PER_THREAD; ++i)
    v_lds_off[i] = (stage_row + i * ROW_STEP) * V_ROW + (((stage_piece >> 1) ^ v_swizzle(stage_row + i * ROW_STEP)) << 5) + ((stage_piece & 1) << 4);

  // Gathering form: every K/V row is fetched through a table of source rows.  For a temporal
  // head row v of the P-outer order is token row_table[entries + v] (Sec. 4.2; text rows map to
  // themselves); a spatial head uses the identity half row_table[v], so that both kinds run the
  // same instructions.  Rows beyond N map to a row outside the tensor, which the bounds-checked
  // loads return as zero.  The entries of a tile are loaded one tile ahead of its K/V rows; a
  // row is 2 D contiguous bytes, so the loads stay whole cache lines.
  const int tab_base = GATHER && pat != 0 ? a.nk * BN * 4 : 0;
  int tab[GATHER ? PER_THREAD : 1];
  auto load_table = [&](int col_any) {
    const int key0 = __builtin_amdgcn_readfirstlane(col_any) * BN;
    const __amdgpu_buffer_rsrc_t rt = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<int32_t*>(a.row_table), 0, 2u * (unsigned)a.nk * BN * 4u, kRsrcFlags);
    if constexpr (GATHER && PER_THREAD == 4) {
      const u32x4 e = __builtin_amdgcn_raw_buffer_load_b128(rt, stage_row * 4, tab_base + key0 * 4, 0);
#pragma unroll
      for (int i = 0; i < 4; ++i) tab[i] = (int)e[i];
    } else if constexpr (GATHER) {
      static_assert(!GATHER || PER_THREAD == 4 || PER_THREAD == 2, "one load fetches a thread's row numbers");
      const u32x2 e = __builtin_amdgcn_raw_buffer_load_b64(rt, stage_row * 4, tab_base + key0 * 4, 0);
      tab[0] = (int)e[0];
      tab[1] = (int)e[1];
    }
  };

  auto load_tile = [&](int col_any) {
    if constexpr (GATHER) {
      const unsigned head_bytes = (unsigned)a.N * (D * 2);
      const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(const_cast<__bf16*>(kh), 0, head_bytes, kRsrcFlags);
      const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(const_cast<__bf16*>(vh), 0, head_bytes, kRsrcFlags);
#pragma unroll
      for (int i = 0; i < PER_THREAD; ++i)
        kst[i] = __builtin_amdgcn_raw_buffer_load_b128(rk, tab[i] * (D * 2) + stage_piece * 16, 0, 0);
#pragma unroll
      for (int i = 0; i < PER_THREAD; ++i)
        vst[i] = __builtin_amdgcn_raw_buffer_load_b128(rv, tab[i] * (D * 2) + stage_piece * 16, 0, 0);
      return;
    }
    // the tile index is the same in every lane; saying so keeps the descriptors scalar
    const int key0 = __builtin_amdgcn_readfirstlane(col_any) * BN;
    const unsigned bytes_left = (unsigned)(a.N - key0) * (D * 2);
    const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<__bf16*>(kh + (size_t)key0 * D), 0, bytes_left, kRsrcFlags);
    const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<__bf16*>(vh + (size_t)key0 * D), 0, bytes_left, kRsrcFlags);
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i)
      kst[i] = __builtin_amdgcn_raw_buffer_load_b128(rk, stage_off + i * ROW_STEP * (D * 2), 0, 0);
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i)
      vst[i] = __builtin_amdgcn_raw_buffer_load_b128(rv, stage_off + i * ROW_STEP * (D * 2), 0, 0);
  };

  auto store_tile = [&](int buf, int col) {
    unsigned char* kb = lds + buf * STAGE_BYTES;
    unsigned char* vb = kb + K_BYTES;
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i)
      *reinterpret_cast<u32x4*>(kb + k_lds_off + i * ROW_STEP * K_ROW) = kst[i];
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i)
      *reinterpret_cast<u32x4*>(vb + v_lds_off[i]) = vst[i];
    if (MASKABLE && masked && tid < BN) {
      // per-key mask code: the key's frame (spatial) or in-frame position (temporal), or
      // "kept by every query" (text / sink key, unmasked pass), or "out of range"
      const int key = col * BN + tid;
      int code;
      if (key >= a.N) {
        code = kCodeDrop;
      } else if ((MODE == kProfile && variant == 0) || key < a.off || key >= a.video_end) {
        code = kCodeKeep;
      } else if (MODE == kSparseExact) {
        // spatial: the key's frame; temporal (transformed order): its in-frame position
        unsigned pk, fk;
        if (pat) {
          transformed_to_token((unsigned)(key - a.off), (unsigned)a.F, (unsigned)a.P, a.sink, &pk, &fk);
        } else {
          fk = (unsigned)(key - a.off) / (unsigned)a.P;
          pk = fk;
        }
        code = (int)pk;
        if (a.sink && fk == 0) code = kCodeKeep;
      } else {
        const int vk = key - a.off;
        const int fk = vk / a.P;
        code = variant == 1 ? fk : vk - fk * a.P;
        if (a.sink && fk == 0) code = kCodeKeep;
      }
      key_code[buf * BN + tid] = code;
      // Summary of the tile for the wave-uniform shortcuts in the masking step.  The
      // coordinate codes of consecutive keys ascend (frames) or ascend by one with a
      // wrap at frame ends (positions), so first and last coordinate lane bound them.
      const bool is_coord = code != kCodeKeep && code != kCodeDrop;
      const unsigned long long coord_lanes = __builtin_amdgcn_ballot_w64(is_coord);
      int flags = (__builtin_amdgcn_ballot_w64(code == kCodeKeep) != 0 ? 1 : 0) |
                  (__builtin_amdgcn_ballot_w64(code == kCodeDrop) != 0 ? 2 : 0);
      int cmin = 0, cmax = -1;          // empty coordinate range
      if (coord_lanes != 0) {
        const int first = __builtin_ctzll(coord_lanes), last = 63 - __builtin_clzll(coord_lanes);
        cmin = __builtin_amdgcn_readlane(code, first);
        cmax = __builtin_amdgcn_readlane(code, last);
        // (positions in frame-major order wrap at frame ends; the coordinates of the exact
        // sparse form never decrease, so first and last always bound them)
        if (MODE == kProfile && variant == 2 && cmax - cmin != last - first) flags |= 4;    // wrapped: treat as mixed
      }
      if (tid == 0) {
        tile_info[buf * 4 + 0] = cmin;
        tile_info[buf * 4 + 1] = cmax;
        tile_info[buf * 4 + 2] = flags;
      }
    }
  };

  // ======================================================================================
  // Main loop.
  // ======================================================================================
  f32x16 oacc[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[db][e] = 0.f;
  float m_run = kNegBig;   // reference maximum (raw logits, before scaling)
  float l_run = 0.f;       // this lane's share of the running row sum

  // a ring holds the current tile and the next three, so no scalar load sits between one
  // tile's barrier and the next tile's global loads
  int col = next_tile(), col1 = next_tile(), col2 = next_tile(), col3 = next_tile();
  if (col != kNoTile) {
    if (GATHER) load_table(col);
    load_tile(col);
    store_tile(0, col);
  }
  if (GATHER && col1 != kNoTile) load_table(col1);
  __syncthreads();

  // Touch Q here so that its loads are known to have completed before the loop.  Without
  // this the compiler's wait-count bookkeeping still sees them pending at the loop head
  // and emits vmcnt waits in front of the first products of every iteration, which then
  // wait for the NEXT tile's freshly issued global loads instead.
#pragma unroll
  for (int s = 0; s < DS; ++s) asm volatile("" ::"v"(qreg[s]));

  int buf = 0;
  // V^T operand reads: this lane's source address inside a 16-key step for channel block db.  As
  // a source lane of the transposing read, lane 16 q + s of the wavefront (q = 2 g + h) supplies
  // the 8 bytes of row 4 g + s / 4 at channel 32 db + 16 h + 4 (s % 4).
  int v_off[DB];
  {
    const int s = lane & 15, j = s >> 2, h = (lane >> 4) & 1;
#pragma unroll
    for (int db = 0; db < DB; ++db)
      v_off[db] = (4 * g + j) * V_ROW + (((2 * db + h) ^ v_swizzle(j)) << 5) + ((s & 3) << 3);
  }
  const bool ragged = (a.N % BN) != 0;

  while (col != kNoTile) {
    const int next_col = col1;
    col1 = col2;
    col2 = col3;
    fetch_begin();
    if (next_col != kNoTile) load_tile(next_col);
    if (GATHER && col1 != kNoTile) load_table(col1);      // entries of the tile after it
    const int tile = col;          // key tile of this iteration

    // profile: does this wavefront need the tile at all, and does it need per-element masks?
    // (a lane whose row keeps none of the tile's keys while other lanes do needs no element masks
    // either: it takes its exponentials against +inf, i.e. all weights zero)
    bool skip = false, need_masks = MASKABLE && masked, drop_lane = false;
    if (MASKABLE && masked) {
      const int cmin = tile_info[buf * 4 + 0], cmax = tile_info[buf * 4 + 1], flags = tile_info[buf * 4 + 2];
      bool lane_all = (flags & 6) == 0, lane_none = (flags & 5) == 0;
      if (cmax >= cmin) {       // the tile has coordinate keys
        const bool in_lo = (unsigned)(cmin - win_lo) <= win_span;
        const bool in_hi = (unsigned)(cmax - win_lo) <= win_span;
        lane_all = lane_all && in_lo && in_hi;
        // disjoint: the whole range lies below or above this row's window
        const long long lo = win_lo, hi = lo + (long long)win_span;
        lane_none = lane_none && (cmax < lo || cmin > hi);
      }
      skip = __builtin_amdgcn_ballot_w64(!lane_none) == 0;   // no row of this wave keeps any key
      need_masks = __builtin_amdgcn_ballot_w64(!lane_all && !lane_none) != 0;   // some row keeps a part of them
      drop_lane = !need_masks && lane_none;
    }

    if (!skip) {
      const unsigned char* kbuf = lds + buf * STAGE_BYTES;
      const unsigned char* vbuf = kbuf + K_BYTES;

      // ---- S^T = K Q^T.  Operand reads run PF products ahead of their use (a rolling
      // window of PF operand registers), so after the first few the LDS latency is hidden
      // behind the MFMAs; the scheduling barriers pin the read / product interleave.
      constexpr int PF = prefetch_depth(D, NW, MODE);
      constexpr int NS = KB * DS;          // operands of the first product, order (kb, s)
      constexpr int NV = KB * 2 * DB;      // operands of the second product, order (kb, kk, db)
      auto k_operand = [&](int i) -> bf16x8 {
        const int kb = i / DS, s = i % DS;
        return *reinterpret_cast<const bf16x8*>(kbuf + (kb * 32 + r) * K_ROW + ((2 * s + g) << 4));
      };
      auto v_operand = [&](int i) -> bf16x8 {
        const int step = i / DB, db = i % DB;     // step = kb * 2 + kk: rows 16 step .. 16 step + 15
        const unsigned char* src = vbuf + step * 16 * V_ROW + v_off[db];
        const i16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)src);
        const i16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_i16x4*)(src + 8 * V_ROW));
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      };
      f32x16 sacc[KB];
      bf16x8 opnd[PF];
#pragma unroll
      for (int i = 0; i < PF; ++i) opnd[i] = k_operand(i);
      __builtin_amdgcn_s_setprio(kPrioFirstProduct);
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        const int kb = i / DS, s = i % DS;
        const bf16x8 ka = opnd[i % PF];
        __builtin_amdgcn_sched_barrier(0);
        if (s == 0) {
#pragma unroll
          for (int e = 0; e < 16; ++e) sacc[kb][e] = 0.f;
        }
        sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qreg[s], sacc[kb], 0, 0, 0);
        // refill the slot just consumed: next K operand, or (at the tail) the first V^T
        // operands, which then arrive while the softmax runs
        if (i + PF < NS) opnd[i % PF] = k_operand(i + PF);
        else opnd[i % PF] = v_operand(i + PF - NS);
        __builtin_amdgcn_sched_barrier(0);
      }

      __builtin_amdgcn_s_setprio(0);
      // ---- masking.  sacc[kb][4 i + jj] belongs to key  col*BN + 32 kb + 8 i + 4 g + jj.
      if (MASKABLE && masked) {
        if (need_masks) {
#pragma unroll
          for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const i32x4 cc = *reinterpret_cast<const i32x4*>(&key_code[buf * BN + kb * 32 + 8 * i + 4 * g]);
#pragma unroll
              for (int jj = 0; jj < 4; ++jj) {
                const bool keep = ((unsigned)(cc[jj] - win_lo) <= win_span) || cc[jj] == kCodeKeep;
                if (!keep) sacc[kb][4 * i + jj] = -INFINITY;
              }
            }
        }
      } else if (ragged && col == a.nk - 1) {
        int lim = a.N - tile * BN - 4 * g;     // keys with 32 kb + 8 i + jj >= lim are out of range
        // opaque to the optimiser: keeps this rarely taken masking code inside the
        // branch instead of being speculated into every tile
        asm volatile("" : "+v"(lim));
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
              if (kb * 32 + 8 * i + jj >= lim) sacc[kb][4 * i + jj] = -INFINITY;
      }
      // ---- online softmax: one query per lane.
      // Fast path: exponentials are taken against the current reference m_run without
      // looking at the tile's maximum.  That is the same softmax as long as nothing
      // overflows, which the row sum reveals: if any lane's partial sum exceeds
      // kLazySum (or is inf / NaN) the whole wave takes the slow path, which finds the
      // tile maximum, raises the reference, rescales O^T and the running sum, and redoes
      // the tile's exponentials.  With a reference within 2^13 of the true maximum the
      // fp32 sums and bf16 weights lose nothing, and almost every tile after the first
      // few stays on the fast path (no max reduction, no rescale).
      bf16x8 pb[KB][2];
      auto exponentiate = [&](float mc) -> float {
        float l_loc = 0.f;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int kk = 0; kk < 2; ++kk) {
            f32x8 p;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
              p[e] = __builtin_amdgcn_exp2f(__builtin_fmaf(sacc[kb][8 * kk + e], a.scale_log2, -mc));
              if (D != 64) l_loc += p[e];
            }
            pb[kb][kk] = __builtin_convertvector(p, bf16x8);
            if (D == 64) {
              // Head dimension 64 is bound by the softmax's VALU work, so the row sum is taken two
              // weights per instruction: dot products of the packed pairs with (1, 1), i.e. over
              // the ROUNDED weights.  (At D = 128 this was slower: the dot products run on the
              // matrix pipeline and compete with the MFMAs there.)  The pairs are taken by vector
              // shuffles: extracted as 32-bit words of the bit-cast vector, the compiler fed all
              // four dot products the same register.
              const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
              const bf16x8 pv = pb[kb][kk];
              l_loc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pv, pv, 0, 1), ones, l_loc, false);
              l_loc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pv, pv, 2, 3), ones, l_loc, false);
              l_loc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pv, pv, 4, 5), ones, l_loc, false);
              l_loc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(pv, pv, 6, 7), ones, l_loc, false);
            }
          }
        return l_loc;
      };
      float l_loc = exponentiate(MASKABLE && drop_lane ? INFINITY : m_run * a.scale_log2);
      if (__builtin_amdgcn_ballot_w64(!(l_loc <= kLazySum)) != 0) {
        float m_loc = sacc[0][0];
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int e = 0; e < 16; ++e) m_loc = fmaxf(m_loc, sacc[kb][e]);
        m_loc = both_halves_max(m_loc);
        if (MASKABLE && drop_lane) m_loc = -INFINITY;
        const float m_new = fmaxf(m_run, m_loc);
        const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * a.scale_log2);
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int e = 0; e < 16; ++e) oacc[db][e] *= alpha;
        l_loc = exponentiate(MASKABLE && drop_lane ? INFINITY : m_new * a.scale_log2);
      }
      l_run += l_loc;

      // ---- O^T += V^T P^T.  The first PF operands were requested at the end of the first
      // product (slot (NS + i) % PF).
      __builtin_amdgcn_s_setprio(kPrioSecondProduct);
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int kbkk = i / DB, db = i % DB;
        const bf16x8 va = opnd[(NS + i) % PF];
        __builtin_amdgcn_sched_barrier(0);
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[kbkk >> 1][kbkk & 1], oacc[db], 0, 0, 0);
        if (i + PF < NV) opnd[(NS + i) % PF] = v_operand(i + PF);
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    __builtin_amdgcn_s_setprio(0);
    if (next_col != kNoTile) store_tile(buf ^ 1, next_col);
    col3 = fetch_end();
    __syncthreads();
    buf ^= 1;
    col = next_col;
  }

  // ======================================================================================
  // Epilogue: normalise and store.  oacc[db][4 i + jj] = O[query r][32 db + 8 i + 4 g + jj]
  // ======================================================================================
  const float l_tot = both_halves_sum(l_run);
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  if (MODE == kProfile) {
    if (qslot < a.t) {
      // output slots: the parts of the unmasked pass, of the spatial pass, of the temporal pass
      const int slot = variant == 0 ? chunk : a.plan.n_full + (variant - 1) * a.plan.n_masked + chunk;
      float* op = static_cast<float*>(a.o) + (((size_t)slot * a.BH + bh) * a.t + qslot) * D;
      if (g == 0) a.stats[((size_t)slot * a.BH + bh) * a.t + qslot] = make_float2(m_run, l_tot);
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          f32x4 x;
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) x[jj] = oacc[db][4 * i + jj] * inv;
          *reinterpret_cast<f32x4*>(op + db * 32 + 8 * i + 4 * g) = x;
        }
    }
  } else {
    if (qslot < a.N) {
      __bf16* op = static_cast<__bf16*>(a.o) + (head + io_row) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          f32x4 x;
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) x[jj] = oacc[db][4 * i + jj] * inv;
          *reinterpret_cast<bf16x4*>(op + db * 32 + 8 * i + 4 * g) = __builtin_convertvector(x, bf16x4);
        }
    }
  }
}

// Groups the sampled rows by in-frame position for the temporal profiling variant:
// order[] receives the indices 0..t-1 sorted by a coarse position bin (text rows
// first), ascending inside a bin.  One workgroup, counting sort with LDS atomics; the
// atomics leave the order inside a bin to chance, and which rows share a wavefront
// decides where that wavefront renews its reference maximum, i.e. the rounding of the
// results, so every bin is sorted afterwards to make the grouping, and with it every
// output bit, the same on every run.
constexpr int kOrderBins = 2048;
__global__ __launch_bounds__(1024) void profile_order_kernel(const int32_t* rows, int t, int off,
                                                             int video_end, int P, int32_t* order) {
  __shared__ int hist[kOrderBins];
  __shared__ int part[1024];
  const int tid = threadIdx.x;
  auto bin_of = [&](int n) -> int {
    if (n < off || n >= video_end) return 0;
    const int p = (n - off) % P;
    return 1 + (int)(((long long)p * (kOrderBins - 1)) / P);
  };
  for (int i = tid; i < kOrderBins; i += 1024) hist[i] = 0;
  __syncthreads();
  for (int i = tid; i < t; i += 1024) atomicAdd(&hist[bin_of(rows[i])], 1);
  __syncthreads();
  // exclusive scan of the 2048 bins: two per thread, then Hillis-Steele over the pair sums
  const int h0 = hist[2 * tid], h1 = hist[2 * tid + 1];
  part[tid] = h0 + h1;
  __syncthreads();
  for (int step = 1; step < 1024; step <<= 1) {
    const int add = tid >= step ? part[tid - step] : 0;
    __syncthreads();
    part[tid] += add;
    __syncthreads();
  }
  const int base = part[tid] - (h0 + h1);
  hist[2 * tid] = base;
  hist[2 * tid + 1] = base + h0;
  __syncthreads();
  for (int i = tid; i < t; i += 1024) order[atomicAdd(&hist[bin_of(rows[i])], 1)] = i;
  __syncthreads();
  // hist[b] is now the end of bin b; insertion sort of each (short) bin by row index
  for (int b = 2 * tid; b < 2 * tid + 2; ++b) {
    const int s = b == 0 ? 0 : hist[b - 1], e = hist[b];
    for (int i = s + 1; i < e; ++i) {
      const int x = order[i];
      int j = i - 1;
      while (j >= s && order[j] > x) {
        order[j + 1] = order[j];
        --j;
      }
      order[j + 1] = x;
    }
  }
}

// Squared errors of the two masked outputs against the unmasked one (Alg. 1, last
// block), first stage: block (x, bh) sums kErrRows sampled rows of head bh and writes
// one partial pair.  Each of the three outputs of a row is first reassembled from the
// parts its pass was cut into: part r holds its normalised output O_r, its reference
// maximum m_r and its row sum l_r, and O = sum_r w_r O_r / sum_r w_r with
// w_r = l_r * 2^((m_r - max_r m_r) * scale_log2); a part that kept no key of the row has
// l_r = 0.  Text query rows are skipped (both masks keep every key for them, so they
// contribute exactly zero).
constexpr int kErrRows = 16;
constexpr int kMaxSlots = kMaxProfileParts + 2 * 4;
__global__ __launch_bounds__(256) void profile_error_kernel(const float* ws, const float2* stats,
                                                            const int32_t* rows, int BH, int t, int D,
                                                            int n_full, int n_masked, float scale_log2, int off,
                                                            int video_end, float2* partial) {
  // weight[row][slot] = w_r / sum w_r within the slot's pass: one thread per (row, pass)
  __shared__ float weight[kErrRows][kMaxSlots];
  const int bh = blockIdx.y;
  const size_t per = (size_t)t * D;
  const int row0 = blockIdx.x * kErrRows, row1 = min(t, row0 + kErrRows);
  const int slots = n_full + 2 * n_masked;
  if (threadIdx.x < kErrRows * 3) {
    const int rr = threadIdx.x / 3, pass = threadIdx.x % 3, row = row0 + rr;
    const int slot0 = pass == 0 ? 0 : n_full + (pass - 1) * n_masked, parts = pass == 0 ? n_full : n_masked;
    if (row < row1) {
      float m_max = -3.0e38f;
      for (int r = slot0; r < slot0 + parts; ++r) {
        const float2 st = stats[((size_t)r * BH + bh) * t + row];
        if (st.y > 0.f) m_max = fmaxf(m_max, st.x);
      }
      float den = 0.f;
      for (int r = slot0; r < slot0 + parts; ++r) {
        const float2 st = stats[((size_t)r * BH + bh) * t + row];
        const float w = st.y > 0.f ? st.y * __builtin_amdgcn_exp2f((st.x - m_max) * scale_log2) : 0.f;
        weight[rr][r] = w;
        den += w;
      }
      const float inv = den > 0.f ? 1.0f / den : 0.f;
      for (int r = slot0; r < slot0 + parts; ++r) weight[rr][r] *= inv;
    }
  }
  __syncthreads();
  float acc_s = 0.f, acc_t = 0.f;
  for (size_t e = (size_t)row0 * D + threadIdx.x; e < (size_t)row1 * D; e += 256) {
    const int row = (int)(e / D);
    const int n = rows[row];
    if (n < off || n >= video_end) continue;
    const float* wr = weight[row - row0];
    const float* x = ws + (size_t)bh * per + e;       // slot r of this element: x[r * BH * per]
    float f = 0.f, os = 0.f, ot = 0.f;
    for (int r = 0; r < n_full; ++r) f = __builtin_fmaf(wr[r], x[(size_t)r * BH * per], f);
    for (int r = n_full; r < n_full + n_masked; ++r) os = __builtin_fmaf(wr[r], x[(size_t)r * BH * per], os);
    for (int r = n_full + n_masked; r < slots; ++r) ot = __builtin_fmaf(wr[r], x[(size_t)r * BH * per], ot);
    const float ds = f - os, dt = f - ot;
    acc_s = __builtin_fmaf(ds, ds, acc_s);
    acc_t = __builtin_fmaf(dt, dt, acc_t);
  }
  __shared__ float red_s[256], red_t[256];
  red_s[threadIdx.x] = acc_s;
  red_t[threadIdx.x] = acc_t;
  __syncthreads();
  for (unsigned step = 128; step > 0; step >>= 1) {      // fixed order: deterministic
    if (threadIdx.x < step) {
      red_s[threadIdx.x] += red_s[threadIdx.x + step];
      red_t[threadIdx.x] += red_t[threadIdx.x + step];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[(size_t)bh * gridDim.x + blockIdx.x] = make_float2(red_s[0], red_t[0]);
}

// Second stage: MSE_s, MSE_t and the label of one head from its partial sums, added in
// index order (deterministic).  label = spatial iff MSE_s < MSE_t (Alg. 1).
__global__ __launch_bounds__(64) void profile_label_kernel(const float2* partial, int n_partial, int t, int D,
                                                           uint8_t* labels, float* mse) {
  const int bh = blockIdx.x;
  if (threadIdx.x != 0) return;
  float sum_s = 0.f, sum_t = 0.f;
  for (int i = 0; i < n_partial; ++i) {
    const float2 p = partial[(size_t)bh * n_partial + i];
    sum_s += p.x;
    sum_t += p.y;
  }
  const float per = (float)t * (float)D;
  const float ms = sum_s / per, mt = sum_t / per;
  if (mse) {
    mse[2 * bh + 0] = ms;
    mse[2 * bh + 1] = mt;
  }
  labels[bh] = ms < mt ? SVG_HEAD_SPATIAL : SVG_HEAD_TEMPORAL;
}

// rows_total: N for dense / sparse, t for profiling
template <int D, int NW, int BN, int MODE>
int launch_one(AttnArgs a, int rows_total, hipStream_t stream) {
  constexpr int BM = 32 * NW;
  a.nqt = (rows_total + BM - 1) / BM;
  a.total = a.BH * a.nqt;
  const unsigned per_xcd = (unsigned)((a.total + 8 * kCohort - 1) / (8 * kCohort)) * kCohort;   // dense
  if (MODE == kSparse || MODE == kSparseExact || MODE == kSparseGather) a.so = sparse_order(a.BH, a.nqt, BM, a.off, a.video_end, a.N, 32 * (NW == 4 ? waves_per_simd(D, NW, MODE) : 2));
  const unsigned grid = MODE == kProfile ? (unsigned)(8 * a.plan.slots() * ((a.total + 7) / 8))
                        : MODE == kDense ? 8u * per_xcd : sparse_grid(a.so, a.BH);
  (void)hipGetLastError();   // drop any stale error left by earlier runtime calls of the process
  constexpr bool SPARSE_MODE = MODE == kSparse || MODE == kSparseExact || MODE == kSparseGather;
  if (SPARSE_MODE && a.BH > 64)      // label classes over more than one 64-head word
    hipLaunchKernelGGL((attn_kernel<D, NW, BN, MODE, SPARSE_MODE ? kWideLabelWords : 1>), dim3(grid), dim3(64 * NW), 0, stream, a);
  else
    hipLaunchKernelGGL((attn_kernel<D, NW, BN, MODE, 1>), dim3(grid), dim3(64 * NW), 0, stream, a);
  return hip_status(hipGetLastError());
}

template <int MODE>
int dispatch(const Geo& g, const AttnArgs& a, int rows_total, hipStream_t stream) {
  if (g.bm == 128) {
    return g.D == 128 ? launch_one<128, 4, 64, MODE>(a, rows_total, stream)
                      : launch_one<64, 4, 64, MODE>(a, rows_total, stream);
  }
  if constexpr (MODE == kSparseGather) return SVG_ERR_UNSUPPORTED;
  else return g.D == 128 ? launch_one<128, 1, 32, MODE>(a, rows_total, stream)
                         : launch_one<64, 1, 32, MODE>(a, rows_total, stream);
}

// Source rows for the gathering form: table[v] = v (spatial heads), table[entries + v] = token
// row of row v of the P-outer order (text rows: themselves); padding: a row outside the tensor.
__global__ void row_table_kernel(int32_t* table, int entries, int N, int off, int video_end, int F, int P, int sink) {
  const int v = blockIdx.x * blockDim.x + threadIdx.x;
  if (v >= entries) return;
  int same = 0x00ffffff, moved = 0x00ffffff;
  if (v < N) {
    same = v;
    moved = v >= off && v < video_end ? off + (int)transformed_to_token((unsigned)(v - off), (unsigned)F, (unsigned)P, sink) : v;
  }
  table[v] = same;
  table[entries + v] = moved;
}

AttnArgs base_args(const Geo& g, const void* q, const void* k, const void* v, void* o) {
  AttnArgs a = {};
  a.q = static_cast<const __bf16*>(q);
  a.k = static_cast<const __bf16*>(k);
  a.v = static_cast<const __bf16*>(v);
  a.o = o;
  a.N = g.N; a.nk = g.nk; a.BH = g.B * g.H;
  a.scale_log2 = g.scale * 1.4426950408889634f;
  a.off = g.off; a.video_end = g.video_end; a.F = g.F; a.P = g.P;
  a.w_s = g.w_s; a.w_t = g.w_t; a.sink = g.sink;
  return a;
}

}  // namespace

int launch_attention(const Geo& g, const void* q, const void* k, const void* v, const void* k_t, const void* v_t,
                     void* o, const uint8_t* labels, const int32_t* row_ptr_s, const int32_t* col_idx_s,
                     const int32_t* row_ptr_t, const int32_t* col_idx_t, bool sparse,
                     bool qo_token_order, bool element_mask, int32_t* row_table, hipStream_t stream) {
  AttnArgs a = base_args(g, q, k, v, o);
  a.k_t = static_cast<const __bf16*>(k_t);
  a.v_t = static_cast<const __bf16*>(v_t);
  a.labels = labels;
  a.qo_token_order = sparse && qo_token_order ? 1 : 0;
  a.row_ptr[0] = row_ptr_s; a.col_idx[0] = col_idx_s;
  a.row_ptr[1] = row_ptr_t; a.col_idx[1] = col_idx_t;
  if (sparse && row_table) {
    // k and v in token order: build the row table, then the gathering form
    if (element_mask || g.bm != 128) return SVG_ERR_UNSUPPORTED;
    const int entries = g.nk * g.bn;
    (void)hipGetLastError();
    hipLaunchKernelGGL(row_table_kernel, dim3((entries + 255) / 256), dim3(256), 0, stream, row_table, entries, g.N,
                       g.off, g.video_end, g.F, g.P, g.sink);
    const int rc = hip_status(hipGetLastError());
    if (rc != SVG_OK) return rc;
    a.row_table = row_table;
    return dispatch<kSparseGather>(g, a, g.N, stream);
  }
  if (sparse && element_mask) return dispatch<kSparseExact>(g, a, g.N, stream);
  return sparse ? dispatch<kSparse>(g, a, g.N, stream) : dispatch<kDense>(g, a, g.N, stream);
}

int launch_profile(const Geo& g, const void* q, const void* k, const void* v, const int32_t* rows,
                   int t, uint8_t* labels, float* mse, float* workspace, hipStream_t stream) {
  AttnArgs a = base_args(g, q, k, v, workspace);
  a.rows = rows;
  a.t = t;
  // workspace: fp32 outputs [slots][BH][t][D] (parts of the unmasked, the spatial and the
  // temporal pass), statistics float2 [slots][BH][t], partial error sums float2
  // [BH][ceil(t/16)], row order int32 [t]
  a.plan = profile_plan(g, t);
  const int ns = a.plan.slots();
  const int groups = (t + g.bm - 1) / g.bm;
  a.rows_per_group = (t + groups - 1) / groups;
  const size_t out_floats = (size_t)ns * a.BH * t * g.D;
  float2* stats = reinterpret_cast<float2*>(workspace + out_floats);
  const int n_partial = (t + kErrRows - 1) / kErrRows;
  float2* partial = stats + (size_t)ns * a.BH * t;
  int32_t* order = reinterpret_cast<int32_t*>(partial + (size_t)a.BH * n_partial);
  a.stats = stats;
  a.order_t = order;
  (void)hipGetLastError();
  hipLaunchKernelGGL(profile_order_kernel, dim3(1), dim3(1024), 0, stream, rows, t, g.off, g.video_end,
                     g.P, order);
  int rc = hip_status(hipGetLastError());
  if (rc != SVG_OK) return rc;
  rc = dispatch<kProfile>(g, a, t, stream);
  if (rc != SVG_OK) return rc;
  (void)hipGetLastError();
  hipLaunchKernelGGL(profile_error_kernel, dim3(n_partial, a.BH), dim3(256), 0, stream, workspace, stats,
                     rows, a.BH, t, g.D, a.plan.n_full, a.plan.n_masked, a.scale_log2, g.off, g.video_end, partial);
  rc = hip_status(hipGetLastError());
  if (rc != SVG_OK) return rc;
  hipLaunchKernelGGL(profile_label_kernel, dim3(a.BH), dim3(64), 0, stream, partial, n_partial, t, g.D,
                     labels, mse);
  return hip_status(hipGetLastError());
}

}  // namespace svg
