// Reuse branch of Algorithm 2: O = A_cached . V, with the cached map read in
// place from the database (the hit index selects the entry; nothing is
// gathered or copied first).
//
// bf16 path (matrix cores, v_mfma_f32_16x16x32_bf16).  One workgroup = one
// (query, layer, head group, block of 128 map rows).  The product is formed
// transposed, O^T = V^T A^T, so that
//   - the map operand is eight consecutive bf16 of one map row per lane: a
//     plain 16-byte global load straight into the MFMA operand, no LDS;
//   - the V operand comes from an LDS tile that was transposed while staging;
//   - each lane ends up with four consecutive d of one output row.
// Causal maps are exactly zero above the diagonal: 16-row block r only needs
// its first ceil((r+1)/2) blocks of 32 columns.  A wave owns row blocks w and
// 7-w of the 128-row block, which gives every wave the same five column
// blocks on the diagonal chunk (1+4, 1+4, 2+3, 2+3).
//
// Two storage layouts of a map [S][S]:
//   dense   row-major, as computed;
//   packed  only the needed 16 x 32 blocks, row-block-major, each block (1 KiB)
//           stored in MFMA operand order: element (i, 8q+e) of the block at
//           offset (16 q + i) * 8 + e.  A wave's load of one block is then one
//           contiguous KiB, a tile is one contiguous run of 20 KiB (S = 128)
//           instead of 32 KiB with holes, and no 128-byte line is fetched for
//           only half of its bytes.
// HBM-bound: per (query, layer, head) the kernel moves S(S+32) map bytes
// (causal bf16), V once per head group and O once.
#include "common.hpp"
#include "launch.hpp"

namespace ac {

struct ApplyArgs {
  const void* maps;     // [M][L][Hq][tile] (device), or one staged entry
  const int32_t* hit;   // [B] device, or nullptr when q_list is used
  const void* V;
  void* O;
  int32_t M, L, layer_begin, Lc, Hq, Hkv, S;
  int32_t heads_per_wg;  // query heads handled by one workgroup (shares V)
  int32_t n_rblk;        // ceil(S / 128)
  int32_t n_tiles;       // B' * Lc * (Hq / heads_per_wg)
  int32_t fixed_entry;   // >= 0: every listed query uses maps as this single entry
  int32_t n_list;        // number of valid q_list items when fixed_entry >= 0
  int32_t q_list[32];    // queries served by the staged entry
};

__device__ __forceinline__ f32x4 mfma16_bf16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                 __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// PREFETCH: the map pieces of the next (head, chunk) step are requested before the products of
// the current one, so a workgroup that walks several steps always has loads in flight.
template <int D, bool CAUSAL, bool PACKED, bool PREFETCH>
__global__ __launch_bounds__(kThreads, (D == 64 ? (PREFETCH ? 3 : 4) : 2))
void apply_bf16_kernel(const ApplyArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* vt = reinterpret_cast<bf16_t*>(smem);                 // [D][kVtStride]
  bf16_t* ost_all = vt + D * kVtStride;                          // [4][32][D + 4]
  constexpr int OS = D + 4;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kq = lane >> 4;

  // Block id -> (tile, 128-row block R).  The row blocks of one tile share V, and workgroups
  // are handed to the 8 XCDs round-robin by id, so ids that differ by a multiple of 8 (same
  // XCD, same L2) are given to one tile.  Heaviest (last) row block first.
  const int bid = blockIdx.x;
  const int tile = (bid >> 3) / a.n_rblk * 8 + (bid & 7);
  const int R = a.n_rblk - 1 - (bid >> 3) % a.n_rblk;
  if (tile >= a.n_tiles) return;
  const int hgroups = a.Hq / a.heads_per_wg;
  const int hg = tile % hgroups;
  const int l = (tile / hgroups) % a.Lc;
  const int bslot = tile / (hgroups * a.Lc);

  int b, entry;
  if (a.fixed_entry >= 0) {
    b = a.q_list[bslot];
    entry = 0;
  } else {
    b = bslot;
    entry = a.hit[b];
    if (entry < 0 || entry >= a.M) return;   // miss (or invalid index): O[b] untouched
  }

  const int S = a.S, g = a.Hq / a.Hkv;
  const int h0 = hg * a.heads_per_wg;
  const int kvh = h0 / g;
  const int n16 = S >> 4, n32 = S >> 5;
  const size_t tile_elems = PACKED ? (size_t)packed_blocks(S, CAUSAL) * 512 : (size_t)S * S;
  const bf16_t* Vt_src = reinterpret_cast<const bf16_t*>(a.V) +
                         (((size_t)b * a.Lc + l) * a.Hkv + kvh) * (size_t)S * D;
  const bf16_t* A_layer = reinterpret_cast<const bf16_t*>(a.maps) +
                          ((size_t)entry * a.L + (a.layer_begin + l)) * ((size_t)a.Hq * tile_elems);

  const int nloc = min(8, n16 - 8 * R);       // 16-row blocks present in this 128-row block
  const int rA = wave, rB = 7 - wave;         // the two row blocks of this wave
  const bool hasA = rA < nloc, hasB = rB < nloc;
  const int n_chunk = CAUSAL ? R + 1 : (S + kChunk - 1) / kChunk;

  // 16-byte operand piece of (16-row block r, 32-column block cb) for this lane
  auto piece = [&](const bf16_t* At, int r, int cb) -> const u32x4* {
    if (PACKED)
      return reinterpret_cast<const u32x4*>(
          At + (size_t)((CAUSAL ? packed_prefix(r) : r * n32) + cb) * 512 + lane * 8);
    return reinterpret_cast<const u32x4*>(At + (size_t)(16 * r + i16) * S + 32 * cb + 8 * kq);
  };
  // column blocks (of the 128-column chunk c) that row blocks A and B need
  auto steps = [&](int c, int& nA, int& nB) {
    const int nk = min(kChunk, S - c * kChunk) >> 5;
    const bool diag = CAUSAL && c == R;
    nA = hasA ? (diag ? (rA >> 1) + 1 : nk) : 0;
    nB = hasB ? (diag ? (rB >> 1) + 1 : nk) : 0;
  };
  auto issue = [&](const bf16_t* At, int c, u32x4 (&am)[8]) {
    int nA, nB;
    steps(c, nA, nB);
#pragma unroll
    for (int t = 0; t < 8; ++t)
      if (t < nA + nB) {
        const bool inA = t < nA;
        am[t] = *piece(At, 8 * R + (inA ? rA : rB), 4 * c + (inA ? t : t - nA));
      }
  };

  u32x4 am[8], am_next[8];
  if (PREFETCH) issue(A_layer + (size_t)h0 * tile_elems, 0, am_next);
  for (int hl = 0; hl < a.heads_per_wg; ++hl) {
    const int h = h0 + hl;
    const bf16_t* At = A_layer + (size_t)h * tile_elems;
    f32x4 accA[D / 16], accB[D / 16];
#pragma unroll
    for (int db = 0; db < D / 16; ++db) {
      accA[db] = f32x4{0.f, 0.f, 0.f, 0.f};
      accB[db] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    for (int c = 0; c < n_chunk; ++c) {
      int nA, nB;
      steps(c, nA, nB);
      // 1. map pieces: requested first, so that they are in flight while V is staged
      if (PREFETCH) {
#pragma unroll
        for (int t = 0; t < 8; ++t) am[t] = am_next[t];
      } else {
        issue(At, c, am);
      }
      // 2. V^T of this chunk into LDS (once per workgroup; shared by its heads)
      if (hl == 0 || n_chunk > 1) {
        if (c > 0 || hl > 0) __syncthreads();
        stage_v_transposed<D>(Vt_src + (size_t)c * kChunk * D, min(kChunk, S - c * kChunk), vt, tid);
        __syncthreads();
      }
      if (PREFETCH) {
        if (c + 1 < n_chunk) issue(At, c + 1, am_next);
        else if (hl + 1 < a.heads_per_wg) issue(At + tile_elems, 0, am_next);
      }
      // 3. O^T[d][i] += sum_j V^T[d][j] A^T[j][i]
      auto vop = [&](int db, int ks) {
        const u32x2* src = reinterpret_cast<const u32x2*>(vt + (16 * db + i16) * kVtStride +
                                                          32 * ks + 8 * kq);
        u32x2 lo = src[0], hi = src[1];
        return u32x4{lo.x, lo.y, hi.x, hi.y};
      };
      if (nA == 4 && nB == 4) {
        // full chunk: both row blocks need the same four column blocks, so every V^T operand
        // read from LDS feeds two products (LDS bandwidth, not HBM, would bound long rows else)
#pragma unroll
        for (int t = 0; t < 4; ++t)
#pragma unroll
          for (int db = 0; db < D / 16; ++db) {
            const u32x4 v = vop(db, t);
            accA[db] = mfma16_bf16(v, am[t], accA[db]);
            accB[db] = mfma16_bf16(v, am[t + 4], accB[db]);
          }
      } else {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
          if (t < nA) {
#pragma unroll
            for (int db = 0; db < D / 16; ++db) accA[db] = mfma16_bf16(vop(db, t), am[t], accA[db]);
          } else if (t < nA + nB) {
#pragma unroll
            for (int db = 0; db < D / 16; ++db)
              accB[db] = mfma16_bf16(vop(db, t - nA), am[t], accB[db]);
          }
        }
      }
    }

    // 4. result registers: out[row i16 of the block][d = 16 db + 4 kq + v].  Both row blocks go
    // through a wave-private LDS buffer so that global stores are contiguous 16-byte pieces.
    bf16_t* ost = ost_all + wave * (32 * OS);
#pragma unroll
    for (int db = 0; db < D / 16; ++db) {
      u32x2 wa, wb;
      wa.x = pack_bf16(accA[db][0], accA[db][1]);
      wa.y = pack_bf16(accA[db][2], accA[db][3]);
      wb.x = pack_bf16(accB[db][0], accB[db][1]);
      wb.y = pack_bf16(accB[db][2], accB[db][3]);
      *reinterpret_cast<u32x2*>(ost + i16 * OS + 16 * db + 4 * kq) = wa;
      *reinterpret_cast<u32x2*>(ost + (16 + i16) * OS + 16 * db + 4 * kq) = wb;
    }
    // LDS operations of one wave execute in order; only the compiler must keep the order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    bf16_t* Ot = reinterpret_cast<bf16_t*>(a.O) +
                 ((((size_t)b * a.Lc + l) * a.Hq + h) * S + (size_t)R * kChunk) * D;
    constexpr int PIECES = 32 * D / 8;
#pragma unroll
    for (int it = 0; it < PIECES / kWave; ++it) {
      const int p = it * kWave + lane;
      const int row = p / (D / 8), c8 = p % (D / 8);
      const bool low = row < 16;
      if (low ? hasA : hasB) {
        const u32x2* s = reinterpret_cast<const u32x2*>(ost + row * OS + 8 * c8);
        u32x2 x = s[0], y = s[1];
        u32x4 w = {x.x, x.y, y.x, y.y};
        const int lrow = low ? 16 * rA + row : 16 * rB + row - 16;
        // written once, never re-read by this kernel: streaming store
        __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(Ot + (size_t)lrow * D + 8 * c8));
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }
}

// Long sequences (S > 128).  The 16x16x32 matrix instruction runs at half the rate of 32x32x16 on
// this chip (measured 1.3 vs 2.0 PFLOP/s), which does not matter for one 128-column chunk per
// tile but bounds the reuse product once a workgroup walks many full chunks.  Here a wave owns
// one 32-row block of the 128-row block and uses v_mfma_f32_32x32x16_bf16.  Only the diagonal
// chunk is unbalanced (wave w needs 2 (w + 1) of its 8 column steps).
//
// V is not transposed by the ALUs here.  Each 128-key chunk is copied global -> LDS directly
// (global_load_lds_dwordx4, no data registers), row-major, into one of two LDS buffers, so the
// copy of chunk c+1 and the map pieces of chunk c+1 are in flight while chunk c is multiplied;
// the matrix operand is then fetched with the transposing LDS read (ds_read_b64_tr_b16): in a
// group of 16 lanes, lane i supplies the address of four consecutive d of key j(i/4) and lane
// t receives, for ITS d, the four keys j(0..3) -- exactly the operand layout, no shuffles.
// Rows are stored unpadded; 16-byte piece p of key row r sits at position p ^ v_piece_swizzle(r),
// which spreads the 32 lanes one LDS cycle serves over all banks; the copy applies the
// permutation by choosing which global piece each lane fetches.
constexpr int kOutStride = 64 + 4;   // row stride of the 16 x 64 output staging passes

template <int D, bool CAUSAL, bool PACKED>
__global__ __launch_bounds__(kThreads, 2) void apply_bf16_long_kernel(const ApplyArgs a) {
  constexpr int PPR = D / 8;                       // 16-byte pieces per V row
  constexpr int NCOPY = kChunk * PPR / kWave / 4;  // copy instructions per wave and chunk
  __shared__ __attribute__((aligned(16))) bf16_t vb0[kChunk * D];
  __shared__ __attribute__((aligned(16))) bf16_t vb1[kChunk * D];
  // Causal maps at head_dim 64: a workgroup takes a PAIR of row blocks (see below).  Its
  // results then leave through a small wave-private buffer, 16 rows x 64 columns per pass,
  // because the V buffers stay in use.
  constexpr bool PAIRED = CAUSAL && D == 64;
  __shared__ __attribute__((aligned(16))) bf16_t ost_small[PAIRED ? 4 * 16 * kOutStride : 8];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: branches on it stay uniform
  const int il = lane & 31, kh = lane >> 5;

  const int bid = blockIdx.x;
  // PAIRED: row blocks are handled in pairs (n_rblk - 1 - p, then p): under the causal mask
  // their chunk counts add up to n_rblk + 1 for every p, so all workgroups of a launch carry
  // equal work, and the chunk pipeline runs on across the switch (one fill per workgroup, not
  // two): 61 -> 70 % of HBM peak at S = 1024, D = 64.  At D = 128 the V copies, not the short
  // workgroups, are the limit and pairing gains nothing; dense maps have equal work anyway.
  const int n_pairs = PAIRED ? (a.n_rblk + 1) >> 1 : a.n_rblk;
  const int tile = (bid >> 3) / n_pairs * 8 + (bid & 7);
  const int pair = (bid >> 3) % n_pairs;
  if (tile >= a.n_tiles) return;
  const int h = tile % a.Hq;
  const int l = (tile / a.Hq) % a.Lc;
  const int bslot = tile / (a.Hq * a.Lc);
  int b, entry;
  if (a.fixed_entry >= 0) {
    b = a.q_list[bslot];
    entry = 0;
  } else {
    b = bslot;
    entry = a.hit[b];
    if (entry < 0 || entry >= a.M) return;   // miss (or invalid index): O[b] untouched
  }

  const int S = a.S, g = a.Hq / a.Hkv;
  const int n32 = S >> 5;
  const size_t tile_elems = PACKED ? (size_t)packed_blocks(S, CAUSAL) * 512 : (size_t)S * S;
  const bf16_t* Vsrc = uniform_ptr(reinterpret_cast<const bf16_t*>(a.V) +
                                   (((size_t)b * a.Lc + l) * a.Hkv + h / g) * (size_t)S * D);
  const bf16_t* At = uniform_ptr(reinterpret_cast<const bf16_t*>(a.maps) +
                                 (((size_t)entry * a.L + (a.layer_begin + l)) * a.Hq + h) * tile_elems);

  const int R_hi = a.n_rblk - 1 - pair, R_lo = PAIRED ? pair : R_hi;   // heaviest first
  const int n_hi = CAUSAL ? R_hi + 1 : (S + kChunk - 1) / kChunk;
  const int n_total = n_hi + (R_hi != R_lo ? (CAUSAL ? R_lo + 1 : n_hi) : 0);
  // chunk t of the workgroup's walk: its row block and its chunk index within that block
  auto row_block = [&](int t) { return t < n_hi ? R_hi : R_lo; };
  auto chunk_of = [&](int t) { return t < n_hi ? t : t - n_hi; };

  // 16-byte operand piece of column step ks (16 columns, counted from column 0) for this lane:
  // map row 32 rb32 + il, columns 16 ks + 8 kh .. + 8, rb32 = 4 R + wave being this wave's rows
  // (32-bit element offsets from the tile's base, which is uniform over the workgroup: the
  // loads then take a scalar base and one offset register instead of 64-bit lane addresses)
  auto piece_row_of = [&](int R) {
    const int rb32 = 4 * R + wave;
    return PACKED
      ? (unsigned)((CAUSAL ? packed_prefix(2 * rb32 + (il >> 4)) : (2 * rb32 + (il >> 4)) * n32) * 512 +
                   (kh * 16 + (il & 15)) * 8)
      : (unsigned)((32 * rb32 + il) * S + 8 * kh);
  };
  const unsigned piece_row_hi = piece_row_of(R_hi), piece_row_lo = piece_row_of(R_lo);
  // (the column step is uniform over the wave: it goes into the scalar base, the lane's own
  // offset stays one register per row block whatever the step)
  auto piece = [&](int R, int ks) -> const u32x4* {
    const unsigned piece_row = R == R_hi ? piece_row_hi : piece_row_lo;
    const char* step_base = reinterpret_cast<const char*>(At + (size_t)ks * (PACKED ? 256 : 16));
    return reinterpret_cast<const u32x4*>(step_base + 2u * piece_row);   // 32-bit BYTE offset
  };
  // column steps of chunk c this wave needs
  auto steps = [&](int R, int c) {
    if (32 * (4 * R + wave) >= S) return 0;
    const int nk = min(kChunk, S - c * kChunk) >> 4;
    return (CAUSAL && c == R) ? min(nk, 2 * (wave + 1)) : nk;
  };
  auto full = [&](int R, int c) {   // uniform over the workgroup: every wave takes all 8 steps
    return !(CAUSAL && c == R) && S - c * kChunk >= kChunk && 32 * (4 * R + 3) < S;
  };
  // map pieces of chunk c into am.  Every lane loads 8 pieces whatever it needs: a step beyond
  // the wave's last one repeats that last piece (same cache lines, no extra memory traffic,
  // never multiplied), which keeps the loads free of per-wave control flow.
  auto issue = [&](int R, int c, u32x4 (&am)[8]) {
    const int nks = steps(R, c);
    if (nks == 0) return;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) am[ks] = *piece(R, 8 * c + min(ks, nks - 1));
  };
  // copy key rows [128 c, 128 c + nj) of V into buf: instruction k = wave + 4 i fills LDS slots
  // [64 k, 64 k + 64) (slot = row * PPR + position), i.e. rows [k 64/PPR, (k + 1) 64/PPR).
  // Row and position of a lane's slot differ between instructions only by whole multiples of
  // 2048 elements on both sides, so one 32-bit lane offset serves all of them.  Rows past the
  // end of V (ragged last chunk) repeat the last row: finite values that are never multiplied.
  const int slot0 = kWave * wave + lane;
  const unsigned copy_off = (unsigned)((slot0 / PPR) * D + 8 * ((slot0 % PPR) ^ v_piece_swizzle<D>(slot0 / PPR)));
  const bf16_t* vrun = Vsrc;   // chunk after chunk, in order: a running (scalar) source pointer
  auto copy_v = [&](bf16_t* buf, int c) {
    const int nj = min(kChunk, S - c * kChunk);
    const bf16_t* src = vrun;
    vrun += kChunk * D;
    if (nj == kChunk) {
#pragma unroll
      for (int i = 0; i < NCOPY; ++i)
        __builtin_amdgcn_global_load_lds(src + (copy_off + 2048u * i), buf + kWave * 8 * (wave + 4 * i),
                                         16, 0, 0);
    } else {
#pragma unroll
      for (int i = 0; i < NCOPY; ++i) {
        const int slot = slot0 + 4 * kWave * i;
        const int row = slot / PPR, pos = slot % PPR;
        const int src_piece = pos ^ v_piece_swizzle<D>(row);
        __builtin_amdgcn_global_load_lds(src + (size_t)min(row, nj - 1) * D + 8 * src_piece,
                                         buf + kWave * 8 * (wave + 4 * i), 16, 0, 0);
      }
    }
  };

  f32x16 acc[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;

  // transposing operand fetch: rows d = 32 db + il of V^T, contraction slots (kh, e) = key
  // 16 ks + 8 kh + e.  Lane i of a 16-lane group names key row 16 ks + 8 kh + i / 4 (+ 4 for
  // the second half) and the four d starting at 32 db + 16 (il / 16) + 4 (i % 4).  The row's
  // permutation only depends on (key & 3), i.e. not on ks: one element offset per (half, db) is
  // kept in a register and ks enters as a constant.
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  int voff[2][D / 32];
  {
    const int t = lane & 15;
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int db = 0; db < D / 32; ++db) {
        const int j = 8 * kh + 4 * half + (t >> 2);               // key row for ks = 0
        const int d0 = 32 * db + 16 * (il >> 4) + 4 * (t & 3);     // first of this lane's four d
        voff[half][db] = j * D + 8 * ((d0 >> 3) ^ v_piece_swizzle<D>(j)) + (d0 & 7);
      }
  }
  auto vop = [&](const bf16_t* buf, int db, int ks) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3)))*)(buf + voff[0][db] + 16 * ks * D));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3)))*)(buf + voff[1][db] + 16 * ks * D));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    s16x8 w = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, w);
  };
  // Products of chunk c.  The scheduling fences keep the compiler from hoisting every operand
  // read of a chunk in front of the first product (more registers than the file has).
  auto compute = [&](const bf16_t* buf, int R, int c, const u32x4 (&am)[8]) {
    if (full(R, c)) {
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
          acc[db] = mfma_bf16(vop(buf, db, ks), __builtin_bit_cast(bf16x8, am[ks]), acc[db]);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      const int nks = steps(R, c);
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        if (ks < nks) {
#pragma unroll
          for (int db = 0; db < D / 32; ++db)
            acc[db] = mfma_bf16(vop(buf, db, ks), __builtin_bit_cast(bf16x8, am[ks]), acc[db]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  // Software pipeline over chunks, unrolled by two so that buffers and register sets alternate
  // without copies: while chunk c is multiplied out of (vb0, am0), the copy of V chunk c + 1
  // into vb1 and the map pieces of chunk c + 1 into am1 are in flight, and vice versa.
  // publish(): this wave's copies and loads have landed (copies are counted like loads), then
  // the barrier makes every wave's part of the V chunk visible and retires the other buffer.
  auto publish = [&]() {
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
  };
  auto prefetch = [&](bf16_t* buf, int t, u32x4 (&am)[8]) {
    if (t == n_hi) vrun = Vsrc;   // the second row block starts over at the first keys
    copy_v(buf, chunk_of(t));
    issue(row_block(t), chunk_of(t), am);
    __builtin_amdgcn_sched_barrier(0);
  };
  // after the last chunk of a row block: the wave's 32 x D result leaves in 16 x 64 passes
  // through its small private buffer (every global store covers whole 128-byte lines), and
  // the accumulator starts over.  No barrier: the V buffers are not touched.
  auto finish = [&](int t) {
    if (!PAIRED) return;   // one row block per workgroup: stored after the loop, through the V buffers
    if (t + 1 != n_hi && t + 1 != n_total) return;
    const int rb32 = 4 * row_block(t) + wave;
    if (32 * rb32 < S) {
      bf16_t* dst = reinterpret_cast<bf16_t*>(a.O) +
                    ((((size_t)b * a.Lc + l) * a.Hq + h) * S + 32 * rb32) * (size_t)D;
      bf16_t* ost = ost_small + wave * (16 * kOutStride);
#pragma unroll
      for (int rh = 0; rh < 2; ++rh)
#pragma unroll
        for (int dh = 0; dh < D / 64; ++dh) {
          if ((il >> 4) == rh) {
#pragma unroll
            for (int dbp = 0; dbp < 2; ++dbp)
#pragma unroll
              for (int vq = 0; vq < 4; ++vq) {
                const f32x16& r = acc[2 * dh + dbp];
                u32x2 w;
                w.x = pack_bf16(r[4 * vq], r[4 * vq + 1]);
                w.y = pack_bf16(r[4 * vq + 2], r[4 * vq + 3]);
                *reinterpret_cast<u32x2*>(ost + (il & 15) * kOutStride + 32 * dbp + 8 * vq + 4 * kh) = w;
              }
          }
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
          for (int it = 0; it < 2; ++it) {
            const int p = it * kWave + lane;
            const int row = p >> 3, c8 = p & 7;
            const u32x2* sp = reinterpret_cast<const u32x2*>(ost + row * kOutStride + 8 * c8);
            u32x2 lo = sp[0], hi = sp[1];
            __builtin_nontemporal_store(
                u32x4{lo.x, lo.y, hi.x, hi.y},
                reinterpret_cast<u32x4*>(dst + (size_t)(16 * rh + row) * D + 64 * dh + 8 * c8));
          }
          __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
          __builtin_amdgcn_wave_barrier();
        }
    }
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;
  };

  u32x4 am0[8], am1[8];
  prefetch(vb0, 0, am0);
  for (int t = 0; t < n_total; t += 2) {
    publish();
    if (t + 1 < n_total) prefetch(vb1, t + 1, am1);
    compute(vb0, row_block(t), chunk_of(t), am0);
    finish(t);
    if (t + 1 < n_total) {
      publish();
      if (t + 2 < n_total) prefetch(vb0, t + 2, am0);
      compute(vb1, row_block(t + 1), chunk_of(t + 1), am1);
      finish(t + 1);
    }
  }
  if constexpr (!PAIRED) {
    __syncthreads();   // every wave is done with both V buffers: they now stage the output
    const int rb32 = 4 * R_hi + wave;
    if (32 * rb32 < S) {
      bf16_t* dst = reinterpret_cast<bf16_t*>(a.O) +
                    ((((size_t)b * a.Lc + l) * a.Hq + h) * S + 32 * rb32) * (size_t)D;
      bf16_t* ost = ((wave & 2) ? vb1 : vb0) + (wave & 1) * (32 * (D + 4));
      store_tile_bf16<D>(acc, 1.0f, ost, dst, lane);
    }
  }
}

// Dense -> packed conversion of whole tiles (database build).  One workgroup per tile; a
// thread moves 16-byte pieces: piece `lane` of packed block (r, cb) is map row 16 r + lane % 16,
// columns 32 cb + 8 (lane / 16) .. + 8.
__global__ __launch_bounds__(kThreads) void pack_maps_kernel(const bf16_t* __restrict__ dense,
                                                             bf16_t* __restrict__ packed, int S,
                                                             int causal) {
  const int n16 = S >> 4, n32 = S >> 5;
  const int nblk = packed_blocks(S, causal);
  const bf16_t* src = dense + (size_t)blockIdx.x * S * S;
  bf16_t* dst = packed + (size_t)blockIdx.x * nblk * 512;
  const int lane = threadIdx.x & 63;
  const int i16 = lane & 15, kq = lane >> 4;
  for (int r = 0; r < n16; ++r) {
    const int nc = causal ? ((r + 1) + 1) >> 1 : n32;
    const int base = causal ? packed_prefix(r) : r * n32;
    for (int cb = threadIdx.x >> 6; cb < nc; cb += kThreads / kWave) {
      const u32x4 v = *reinterpret_cast<const u32x4*>(src + (size_t)(16 * r + i16) * S + 32 * cb + 8 * kq);
      *reinterpret_cast<u32x4*>(dst + (size_t)(base + cb) * 512 + lane * 8) = v;
    }
  }
}

// fp32 path (vector ALUs): small, correctness-first kernel for fp32 databases (dense layout).
// One workgroup per (query, layer, head); thread t owns outputs (i, d) with
// i*D + d = t, t + 256, ...; sums run over j in ascending order in fp32.
__global__ __launch_bounds__(kThreads) void apply_f32_kernel(const ApplyArgs a, int D, int causal) {
  const int tile = blockIdx.x;
  const int h = tile % a.Hq;
  const int l = (tile / a.Hq) % a.Lc;
  const int bslot = tile / (a.Hq * a.Lc);
  int b, entry;
  if (a.fixed_entry >= 0) {
    b = a.q_list[bslot];
    entry = 0;
  } else {
    b = bslot;
    entry = a.hit[b];
    if (entry < 0 || entry >= a.M) return;
  }
  const int S = a.S, g = a.Hq / a.Hkv;
  const float* A = reinterpret_cast<const float*>(a.maps) +
                   (((size_t)entry * a.L + (a.layer_begin + l)) * a.Hq + h) * (size_t)S * S;
  const float* V = reinterpret_cast<const float*>(a.V) +
                   (((size_t)b * a.Lc + l) * a.Hkv + h / g) * (size_t)S * D;
  float* O = reinterpret_cast<float*>(a.O) + (((size_t)b * a.Lc + l) * a.Hq + h) * (size_t)S * D;
  for (int idx = threadIdx.x; idx < S * D; idx += kThreads) {
    const int i = idx / D, d = idx % D;
    const int nj = causal ? i + 1 : S;
    float acc = 0.f;
    for (int j = 0; j < nj; ++j) acc = fmaf(A[(size_t)i * S + j], V[(size_t)j * D + d], acc);
    O[idx] = acc;
  }
}

static size_t apply_lds_bytes(int D) {
  return (size_t)(D * kVtStride + 4 * 32 * (D + 4)) * sizeof(bf16_t);
}

template <int D, bool CAUSAL, bool PACKED, bool PREFETCH>
static hipError_t launch_bf16(const ApplyArgs& a, dim3 grid, hipStream_t stream) {
  const size_t lds = apply_lds_bytes(D);
  hipError_t e = ensure_lds<&apply_bf16_kernel<D, CAUSAL, PACKED, PREFETCH>>(lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((apply_bf16_kernel<D, CAUSAL, PACKED, PREFETCH>), grid, dim3(kThreads), lds,
                     stream, a);
  return hipGetLastError();
}

template <int D, bool CAUSAL>
static hipError_t launch_bf16_dc(const ApplyArgs& a, dim3 grid, bool packed, bool prefetch,
                                 hipStream_t stream) {
  if (packed) {
    return prefetch ? launch_bf16<D, CAUSAL, true, true>(a, grid, stream)
                    : launch_bf16<D, CAUSAL, true, false>(a, grid, stream);
  }
  return prefetch ? launch_bf16<D, CAUSAL, false, true>(a, grid, stream)
                  : launch_bf16<D, CAUSAL, false, false>(a, grid, stream);
}

template <int D, bool CAUSAL, bool PACKED>
static hipError_t launch_long(const ApplyArgs& a, int tiles8, hipStream_t stream) {
  // causal maps at head_dim 64: a workgroup takes a pair of row blocks (see the kernel)
  const int per_tile = (CAUSAL && D == 64) ? (a.n_rblk + 1) / 2 : a.n_rblk;
  const dim3 grid((unsigned)(tiles8 * per_tile));
  hipLaunchKernelGGL((apply_bf16_long_kernel<D, CAUSAL, PACKED>), grid, dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_long_d(const ApplyArgs& a, int tiles8, bool causal, bool packed,
                                hipStream_t stream) {
  if (causal) return packed ? launch_long<D, true, true>(a, tiles8, stream)
                            : launch_long<D, true, false>(a, tiles8, stream);
  return packed ? launch_long<D, false, true>(a, tiles8, stream)
                : launch_long<D, false, false>(a, tiles8, stream);
}

// Host launcher.  Shapes were validated by the caller (api.hip).
hipError_t launch_apply(const ApplyLaunch& p, hipStream_t stream) {
  ApplyArgs a;
  a.maps = p.maps; a.hit = p.hit; a.V = p.V; a.O = p.O;
  a.M = p.M; a.L = p.L; a.layer_begin = p.layer_begin; a.Lc = p.Lc;
  a.Hq = p.Hq; a.Hkv = p.Hkv; a.S = p.S;
  a.fixed_entry = p.fixed_entry; a.n_list = p.n_list;
  for (int i = 0; i < 32; ++i) a.q_list[i] = i < p.n_list ? p.q_list[i] : 0;
  const int nb = p.fixed_entry >= 0 ? p.n_list : p.B;
  if (nb == 0 || p.Lc == 0) return hipSuccess;

  if (p.is_f32) {
    a.heads_per_wg = 1; a.n_rblk = 1; a.n_tiles = nb * p.Lc * p.Hq;
    hipLaunchKernelGGL(apply_f32_kernel, dim3(a.n_tiles), dim3(kThreads), 0, stream, a, p.D,
                       p.causal);
    return hipGetLastError();
  }
  a.n_rblk = (p.S + kChunk - 1) / kChunk;
  const int g = p.Hq / p.Hkv;
  a.heads_per_wg = (a.n_rblk == 1) ? g : 1;
  a.n_tiles = nb * p.Lc * (p.Hq / a.heads_per_wg);
  const int tiles8 = (a.n_tiles + 7) / 8 * 8;
  const dim3 grid((unsigned)(tiles8 * a.n_rblk));
  if (a.n_rblk > 1)   // long rows: 32-row blocks per wave, full-rate matrix instruction
    return p.D == 64 ? launch_long_d<64>(a, tiles8, p.causal, p.packed, stream)
                     : launch_long_d<128>(a, tiles8, p.causal, p.packed, stream);
  // a workgroup that walks several heads prefetches the next head's map pieces
  const bool prefetch = a.heads_per_wg > 1;
  if (p.D == 64)
    return p.causal ? launch_bf16_dc<64, true>(a, grid, p.packed, prefetch, stream)
                    : launch_bf16_dc<64, false>(a, grid, p.packed, prefetch, stream);
  return p.causal ? launch_bf16_dc<128, true>(a, grid, p.packed, prefetch, stream)
                  : launch_bf16_dc<128, false>(a, grid, p.packed, prefetch, stream);
}

hipError_t launch_pack_maps(const void* dense, void* packed, int64_t n_tiles, int32_t S,
                            int32_t causal, hipStream_t stream) {
  if (n_tiles == 0) return hipSuccess;
  hipLaunchKernelGGL(pack_maps_kernel, dim3((unsigned)n_tiles), dim3(kThreads), 0, stream,
                     reinterpret_cast<const bf16_t*>(dense), reinterpret_cast<bf16_t*>(packed), S,
                     causal);
  return hipGetLastError();
}

}  // namespace ac
