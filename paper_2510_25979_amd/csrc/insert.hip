// Database building on the device (Fig. 3, steps 2 and 3): the recompute branch of Algorithm 2
// for inputs that are to be remembered.  For every selected item the kernel computes
// O = softmax(scale * Q K^T) V like attention_exact, and ALSO writes the normalised map
// A = softmax(scale * Q K^T) of every (layer, head), rounded once to bf16, into the item's slot
// of the map store, in the store's layout; a second small kernel copies the item's feature
// vector into the same slot of the feature store.  A later search that hits the slot makes
// attncache_apply reproduce this O from the stored map.
//
// The map has to be normalised before it is written, so the row statistics must be known before
// the first weight leaves: two passes over the keys.  Pass 1 forms the scores and keeps only the
// row maximum m and the row sum l of 2^(score - m); pass 2 forms the scores again, turns them
// into a = 2^(score - m) / l, rounds to bf16, stores them and multiplies the ROUNDED weights
// with V (so O is exactly what the stored map yields, up to summation order).  Same transposed
// products and register hand-over as the exact kernel: S^T = K Q^T (a lane holds 16 keys of one
// query row), O^T = V^T A^T with A taken from the first product's result registers.
// For S <= 128 K and V are staged in LDS once per group of query heads that share them and both
// passes of every head read them there; longer sequences stream 64-key chunks through two LDS
// stages, once per pass.
//
// Packed layout (see pack_maps_kernel): the result registers of one 32 x 32 score block map onto
// packed 16 x 32 blocks directly -- register group q (4 registers) of lane (row i, half kh) is
// elements 4 kh .. 4 kh + 3 of piece (16 q + i % 16), i.e. one 8-byte store per group, and the 32
// lanes of a 16-row half fill a contiguous 256-byte run.
#include "common.hpp"
#include "launch.hpp"

namespace ac {

struct InsertArgs {
  const void *Q, *K, *V;
  void *O, *maps;
  const int32_t *slot, *row_sel, *key_len;
  int32_t B, M, L, layer_begin, Lc, Hq, Hkv, S;
  int32_t n_rblk, n_tiles;
  int32_t heads_per_wg;   // query heads one workgroup walks (they share K and V)
  float scale_log2e;
};

// One workgroup = one (item, layer, group of query heads that share K and V, 128 query rows),
// walking the keys in chunks of 64 -- twice per head, see above.  K and V reach the matrix cores
// the way they do in the exact kernel: every chunk is copied global -> LDS directly (no data
// registers, no ALU work) into one of two stages, rows unpadded with the 16-byte pieces
// permuted (k_piece_swizzle, v_piece_swizzle), V^T fetched with the transposing LDS read.
//   RESIDENT (S <= 128): both chunks sit in the two stages for the whole tile and the workgroup
//   walks all g query heads of the group -- K and V come from HBM once per group, and after the
//   one barrier behind the copy the four waves never meet again.
//   Streaming (S > 128): one head per workgroup; the copy of chunk c + 1 is in flight while chunk
//   c is multiplied, one barrier per chunk; the statistics pass needs no V and copies none.
constexpr int kIChunk = 64;   // keys per staged chunk

template <int D, bool CAUSAL, bool PACKED, bool RESIDENT>
__global__ __launch_bounds__(kThreads, 2) void insert_bf16_kernel(const InsertArgs a) {
  constexpr int PPR = D / 8;                          // 16-byte pieces per row
  constexpr int NCOPY = kIChunk * PPR / kWave / 4;    // copy instructions per wave, tensor, chunk
  __shared__ __attribute__((aligned(16))) bf16_t kb0[kIChunk * D];
  __shared__ __attribute__((aligned(16))) bf16_t vb0[kIChunk * D];
  __shared__ __attribute__((aligned(16))) bf16_t kb1[kIChunk * D];
  __shared__ __attribute__((aligned(16))) bf16_t vb1[kIChunk * D];
  __shared__ __attribute__((aligned(16))) bf16_t ost_small[4 * 16 * kSmallOutStride];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int il = lane & 31, kh = lane >> 5;
  const int S = a.S, g = a.Hq / a.Hkv;

  // same id scheme as above: all row blocks of a head, and all heads that share K and V, get
  // ids equal mod 8 (one XCD, one L2).  RESIDENT (S <= 128): both chunks of K and V sit in the
  // two stages for the whole tile and the workgroup walks all heads_per_wg = g query heads
  // that share them; between the one barrier after the copy and the end of the tile the four
  // waves never meet again.
  const int bid = blockIdx.x;
  const int hslots = g / a.heads_per_wg;
  const int slot_id = bid >> 3;
  const int grp = (slot_id / (hslots * a.n_rblk)) * 8 + (bid & 7);   // (item, layer, KV head)
  const int hslot = (slot_id / a.n_rblk) % hslots;
  const int R = a.n_rblk - 1 - slot_id % a.n_rblk;
  if (grp >= a.n_tiles) return;
  const int kvh = grp % a.Hkv;
  const int l = (grp / a.Hkv) % a.Lc;
  const int b = grp / (a.Hkv * a.Lc);
  if (a.row_sel && a.row_sel[b] >= 0) return;
  const int len = a.key_len ? min(max(a.key_len[b], 1), S) : S;
  const int entry = a.slot ? a.slot[b] : -1;
  const bool keep = entry >= 0 && entry < a.M;   // anything else: compute O only

  const size_t kv = (((size_t)b * a.Lc + l) * a.Hkv + kvh) * (size_t)S * D;
  const bf16_t* Ksrc = reinterpret_cast<const bf16_t*>(a.K) + kv;
  const bf16_t* Vsrc = reinterpret_cast<const bf16_t*>(a.V) + kv;
  const int n_all = (S + kIChunk - 1) / kIChunk;
  const int n_chunk = CAUSAL ? min(2 * (R + 1), n_all) : n_all;   // the same for all four waves
  const int r0 = R * kChunk + 32 * wave;
  const bool active = r0 < S;
  const int n32 = S >> 5;
  const size_t tile_elems = PACKED ? (size_t)packed_blocks(S, CAUSAL) * 512 : (size_t)S * S;
  bf16_t* At = nullptr;   // the current head's map in the store

  // ---- copies: instruction k = wave + 4 i fills LDS slots [64 k, 64 k + 64), slot = row * PPR +
  // position; from one instruction to the next the row grows by 256 / PPR, which leaves both
  // permutations unchanged.  Rows past the end of a ragged last chunk repeat its last row
  // (finite, and never multiplied: the block count below stops before them).
  const int slot0 = kWave * wave + lane;
  const int crow = slot0 / PPR, cpos = slot0 % PPR;
  const int kpiece = cpos ^ k_piece_swizzle<D>(crow);
  const int vpiece = cpos ^ v_piece_swizzle<D>(crow);
  auto prefetch = [&](bf16_t* kb, bf16_t* vb, int c, const bool WITH_V) {
    const int nj = min(kIChunk, S - c * kIChunk);
    const bf16_t* ksrc = Ksrc + (size_t)c * kIChunk * D;
    const bf16_t* vsrc = Vsrc + (size_t)c * kIChunk * D;
#pragma unroll
    for (int i = 0; i < NCOPY; ++i) {
      const int rr = min(crow + (256 / PPR) * i, nj - 1);
      __builtin_amdgcn_global_load_lds(ksrc + (size_t)rr * D + 8 * kpiece,
                                       kb + kWave * 8 * (wave + 4 * i), 16, 0, 0);
      if (WITH_V)
        __builtin_amdgcn_global_load_lds(vsrc + (size_t)rr * D + 8 * vpiece,
                                         vb + kWave * 8 * (wave + 4 * i), 16, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  // this wave's copies have landed (they are counted like loads), then everybody's; the
  // barrier also retires the stage that the next copy overwrites
  auto publish = [&]() {
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
  };

  // ---- operand addresses (elements, relative to a stage), as in the exact kernel
  int koff[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) koff[ks] = il * D + 8 * ((2 * ks + kh) ^ k_piece_swizzle<D>(il));
  typedef short s16x4 __attribute__((ext_vector_type(4)));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  int voff[2][D / 32];
  {
    const int t = lane & 15;
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
      for (int db = 0; db < D / 32; ++db) {
        const int j = 4 * kh + 8 * half + (t >> 2);
        const int d0 = 32 * db + 16 * (il >> 4) + 4 * (t & 3);
        voff[half][db] = j * D + 8 * ((d0 >> 3) ^ v_piece_swizzle<D>(j)) + (d0 & 7);
      }
  }
  // V^T operand of contraction step s2 of key block jb: slot e of lane half kh is key
  // 16 s2 + 8 (e / 4) + 4 kh + e % 4 of the block, where the first product left the scores
  auto vop = [&](const bf16_t* vb, int db, int jb, int s2) {
    const int base = (32 * jb + 16 * s2) * D;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3)))*)(vb + voff[0][db] + base));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (s16x4 __attribute__((address_space(3)))*)(vb + voff[1][db] + base));
    s16x8 w = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, w);
  };

  u32x4 q[D / 16];
  // 32-key blocks of chunk c this wave's rows see
  auto blocks = [&](int c) {
    if (!active) return 0;
    const int j0 = c * kIChunk;
    int nblk = min(kIChunk, S - j0) >> 5;
    if (CAUSAL) nblk = min(nblk, (r0 - j0) / 32 + 1);
    return max(nblk, 0);
  };
  // scores^T of key block jb of the staged chunk c (keys beyond the diagonal or in the padding
  // hidden; the first block of a row always has a visible key, so the running maximum is
  // finite from then on)
  auto scores = [&](const bf16_t* kb, int c, int jb) {
    f32x16 s;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks)
      s = mfma_bf16(*reinterpret_cast<const bf16x8*>(kb + koff[ks] + 32 * jb * D),
                    __builtin_bit_cast(bf16x8, q[ks]), s);
    const int j00 = c * kIChunk + 32 * jb;
    if ((CAUSAL && j00 == r0) || j00 + 32 > len) {   // wave-uniform: most blocks skip the tests
      int limit = len - 1 - j00;
      if (CAUSAL) limit = min(limit, r0 + il - j00);
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (mfma_row(v, kh) > limit) s[v] = -INFINITY;
    }
    return s;
  };

  float m_run = -INFINITY, l_run = 0.f, inv_l = 0.f;
  f32x16 acc[D / 32];
  // where register group q4 (scores 4 q4 .. 4 q4 + 3 of this lane) of 32-key block kb goes
  const int r16 = (r0 >> 4) + (il >> 4);
  auto map_piece = [&](int kb, int q4) -> u32x2* {
    if (PACKED) {
      const int blk = (CAUSAL ? packed_prefix(r16) : r16 * n32) + kb;
      return reinterpret_cast<u32x2*>(At + (size_t)blk * 512 + (16 * q4 + (il & 15)) * 8 + 4 * kh);
    }
    return reinterpret_cast<u32x2*>(At + (size_t)(r0 + il) * S + 32 * kb + 8 * q4 + 4 * kh);
  };

  // one staged chunk.  First pass: row maximum m (log2 domain, scale folded in) and row sum l of
  // 2^(score - m).  Second pass: normalised weights, rounded, stored, multiplied with V.
  auto chunk = [&](const bf16_t* kb, const bf16_t* vb, int c, const bool SECOND)
                   __attribute__((always_inline)) {
    const int nblk = blocks(c);
    for (int jb = 0; jb < nblk; ++jb) {
      f32x16 s = scores(kb, c, jb);
      if (!SECOND) {
        float mx = s[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[v]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx * a.scale_log2e);
        float psum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) psum += __builtin_amdgcn_exp2f(fmaf(s[v], a.scale_log2e, -m_new));
        l_run = l_run * __builtin_amdgcn_exp2f(m_run - m_new) + psum;
        m_run = m_new;
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v)
          s[v] = __builtin_amdgcn_exp2f(fmaf(s[v], a.scale_log2e, -m_run)) * inv_l;
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          u32x4 pw;
          pw.x = pack_bf16(s[8 * s2 + 0], s[8 * s2 + 1]);
          pw.y = pack_bf16(s[8 * s2 + 2], s[8 * s2 + 3]);
          pw.z = pack_bf16(s[8 * s2 + 4], s[8 * s2 + 5]);
          pw.w = pack_bf16(s[8 * s2 + 6], s[8 * s2 + 7]);
          if (keep) {
            const int kb32 = 2 * c + jb;
            *map_piece(kb32, 2 * s2) = u32x2{pw.x, pw.y};
            *map_piece(kb32, 2 * s2 + 1) = u32x2{pw.z, pw.w};
          }
          const bf16x8 pop = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
          for (int db = 0; db < D / 32; ++db) acc[db] = mfma_bf16(vop(vb, db, jb, s2), pop, acc[db]);
        }
      }
    }
  };
  // all chunks of the row block, two per trip so that the stages are named statically (the
  // compiler then knows that the copy in flight and the reads of the other stage do not meet)
  auto pass = [&](const bool SECOND) __attribute__((always_inline)) {
    prefetch(kb0, vb0, 0, SECOND);
    publish();
    int c = 0;
    for (; c + 1 < n_chunk; c += 2) {
      prefetch(kb1, vb1, c + 1, SECOND);
      chunk(kb0, vb0, c, SECOND);
      publish();
      if (c + 2 < n_chunk) prefetch(kb0, vb0, c + 2, SECOND);
      chunk(kb1, vb1, c + 1, SECOND);
      publish();
    }
    if (c < n_chunk) {   // odd count: the last chunk sits in the first stage
      chunk(kb0, vb0, c, SECOND);
      publish();         // everybody is done with it before the next pass overwrites it
    }
  };

  if (RESIDENT) {
    prefetch(kb0, vb0, 0, true);
    if (n_chunk > 1) prefetch(kb1, vb1, 1, true);
    publish();
  }
  const int n_heads = RESIDENT ? a.heads_per_wg : 1;   // streaming: one head per workgroup
  for (int hl = 0; hl < n_heads; ++hl) {
    const int h = kvh * g + hslot * a.heads_per_wg + hl;
    const size_t qo = (((size_t)b * a.Lc + l) * a.Hq + h) * (size_t)S * D;
    At = reinterpret_cast<bf16_t*>(a.maps) +
         (((size_t)(keep ? entry : 0) * a.L + (a.layer_begin + l)) * a.Hq + h) * tile_elems;
    if (active) {
      const bf16_t* qrow = reinterpret_cast<const bf16_t*>(a.Q) + qo + (size_t)(r0 + il) * D + 8 * kh;
#pragma unroll
      for (int ks = 0; ks < D / 16; ++ks) q[ks] = *reinterpret_cast<const u32x4*>(qrow + 16 * ks);
    }
    m_run = -INFINITY;
    l_run = 0.f;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;

    if (RESIDENT) {
      chunk(kb0, vb0, 0, false);
      if (n_chunk > 1) chunk(kb1, vb1, 1, false);
      inv_l = 1.0f / (l_run + __shfl_xor(l_run, 32));
      chunk(kb0, vb0, 0, true);
      if (n_chunk > 1) chunk(kb1, vb1, 1, true);
    } else {
      pass(false);
      inv_l = 1.0f / (l_run + __shfl_xor(l_run, 32));
      pass(true);
    }

    if (active) {
      // A dense causal map carries its zeros: the 32-column blocks right of the diagonal block
      // (the packed layout does not store them)
      if (CAUSAL && !PACKED && keep) {
        for (int kb = (r0 >> 5) + 1; kb < n32; ++kb)
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) *map_piece(kb, q4) = u32x2{0u, 0u};
      }
      // the result leaves through the wave's small buffer: K and V stay where they are
      bf16_t* Oh = reinterpret_cast<bf16_t*>(a.O) + qo + (size_t)r0 * D;
      store_tile_bf16_small<D>(acc, 1.0f, ost_small + wave * (16 * kSmallOutStride), Oh, lane);
    }
  }
}

// feature vector of item b into row slot[b] of the feature store (16-byte pieces)
__global__ __launch_bounds__(kThreads) void insert_features_kernel(const u32x4* __restrict__ feat,
                                                                   u32x4* __restrict__ emb,
                                                                   const int32_t* __restrict__ slot,
                                                                   const int32_t* __restrict__ row_sel,
                                                                   int32_t M, int32_t pieces) {
  const int b = blockIdx.x;
  if (row_sel && row_sel[b] >= 0) return;
  const int entry = slot[b];
  if (entry < 0 || entry >= M) return;
  for (int p = threadIdx.x; p < pieces; p += kThreads)
    emb[(size_t)entry * pieces + p] = feat[(size_t)b * pieces + p];
}

template <int D, bool CAUSAL, bool PACKED>
static hipError_t launch_insert_t(const InsertArgs& a, dim3 grid, hipStream_t stream) {
  if (a.n_rblk == 1)
    hipLaunchKernelGGL((insert_bf16_kernel<D, CAUSAL, PACKED, true>), grid, dim3(kThreads), 0, stream, a);
  else
    hipLaunchKernelGGL((insert_bf16_kernel<D, CAUSAL, PACKED, false>), grid, dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

template <int D>
static hipError_t launch_insert_d(const InsertArgs& a, dim3 grid, bool causal, bool packed,
                                       hipStream_t stream) {
  if (causal) return packed ? launch_insert_t<D, true, true>(a, grid, stream)
                            : launch_insert_t<D, true, false>(a, grid, stream);
  return packed ? launch_insert_t<D, false, true>(a, grid, stream)
                : launch_insert_t<D, false, false>(a, grid, stream);
}

// Host launcher.  Shapes were validated by the caller (api.hip).
hipError_t launch_insert(const InsertLaunch& p, hipStream_t stream) {
  if (p.B == 0 || p.Lc == 0) return hipSuccess;
  if (p.feat) {
    hipLaunchKernelGGL(insert_features_kernel, dim3((unsigned)p.B), dim3(kThreads), 0, stream,
                       reinterpret_cast<const u32x4*>(p.feat), reinterpret_cast<u32x4*>(p.emb),
                       p.slot, p.row_sel, p.M, p.emb_row_bytes / 16);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  InsertArgs a;
  a.Q = p.Q; a.K = p.K; a.V = p.V; a.O = p.O; a.maps = p.maps;
  a.slot = p.slot; a.row_sel = p.row_sel; a.key_len = p.key_len;
  a.B = p.B; a.M = p.M; a.L = p.L; a.layer_begin = p.layer_begin; a.Lc = p.Lc;
  a.Hq = p.Hq; a.Hkv = p.Hkv; a.S = p.S;
  a.n_rblk = (p.S + kChunk - 1) / kChunk;
  a.n_tiles = p.B * p.Lc * p.Hkv;   // KV groups: (item, layer, KV head)
  const float scale = p.scale == 0.f ? 1.0f / sqrtf((float)p.D) : p.scale;
  a.scale_log2e = scale * 1.44269504088896340736f;
  const int g = p.Hq / p.Hkv;
  a.heads_per_wg = a.n_rblk == 1 ? g : 1;
  const int groups8 = (a.n_tiles + 7) / 8 * 8;   // padded to a multiple of 8
  const dim3 grid((unsigned)((size_t)groups8 * (g / a.heads_per_wg) * a.n_rblk));
  return p.D == 64 ? launch_insert_d<64>(a, grid, p.causal, p.packed, stream)
                   : launch_insert_d<128>(a, grid, p.causal, p.packed, stream);
}

}  // namespace ac
