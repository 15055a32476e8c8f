// Recompute branch of Algorithm 2: O = softmax(scale * Q K^T) V, causal or
// dense, without ever writing the S x S map (flash-style online softmax).
//
// bf16 path (matrix cores, v_mfma_f32_32x32x16_bf16), one kernel in two variants:
//   * resident (S <= 128): one workgroup = one (batch item, KV head); both 64-key chunks of K
//     and V are copied into LDS once and the workgroup walks all g query heads that share
//     them; after the one barrier behind the copy its four waves never meet again;
//   * streaming (S > 128): one workgroup = one (batch item, query head, block of 128 query
//     rows) that streams 64-key chunks of K and V through two LDS stages.
// A wave owns 32 query rows and walks the key blocks up to its diagonal.
// Both products are formed transposed:
//   S^T = K Q^T   -> a lane holds 16 keys of ONE query column, so the row
//                    maximum and row sum are in-lane reductions plus one
//                    exchange between the two lane halves;
//   O^T = V^T P^T -> the probabilities sit in exactly the register layout
//                    the second product wants as its column operand, so P
//                    goes from the first MFMA to the second without leaving
//                    registers (the contraction slots are matched by reading
//                    V^T from LDS in the same key order).
// Softmax runs in the log2 domain with the scale folded into one FMA per
// score; the accumulator is rescaled only when some row maximum has moved far.
#include "common.hpp"
#include "launch.hpp"

namespace ac {

constexpr int kOPass = 64; // output columns staged per pass (16 rows at a time)
constexpr int kOStride = kOPass + 4;
// Online softmax: weights are 2^(score - m); m moves (and the accumulator is rescaled) only when
// a row maximum has outgrown it by more than this many bits (see the chunk step below).
constexpr float kRescaleSlack = 8.0f;

struct ExactArgs {
  const void *Q, *K, *V;
  void* O;
  const int32_t* row_sel;
  const int32_t* key_len;   // real tokens per batch item of a right-padded batch, or nullptr
  int32_t B, Hq, Hkv, S;
  int32_t heads_per_wg;
  int32_t n_rblk;
  int32_t n_kvtiles;
  int32_t n_blocks;   // tiles of the launch (the grid of a routed resident launch is smaller)
  float scale_log2e;
};

// How K and V reach the matrix cores:
//   * each chunk of K and of V is copied global -> LDS directly (global_load_lds_dwordx4, no
//     data registers, no ALU work), row-major, into one of two stages, so the copy of chunk
//     c + 1 is in flight while chunk c is multiplied and one barrier per chunk suffices;
//   * rows are unpadded; the copy permutes the 16-byte pieces of a row (a lane picks which
//     global piece lands in its LDS slot) so that the operand reads spread over all banks:
//     K piece p of row r sits at p ^ k_piece_swizzle(r), V piece p of row r at p ^ v_piece_swizzle(r);
//   * the V^T operand is fetched with the transposing LDS read (ds_read_b64_tr_b16): in a
//     group of 16 lanes, lane i names four consecutive d of key j(i / 4) and lane t receives,
//     for its own d, the four keys j(0..3);
//   * the two 32-key blocks of a chunk take their softmax steps in an order that lets matrix
//     and vector work of one wave overlap (see the chunk step below).
constexpr int kLChunk = 64;

// max(x[l], x[l ^ 32]) in every lane l.  v_permlane32_swap_b32 exchanges the upper 32 lanes of
// its first register with the lower 32 lanes of its second one, so two copies of x become
// (lower half twice) and (upper half twice) without a trip through LDS.  Written as inline
// assembly because the compiler builtin of the same name folds its two results into one in
// this toolchain; the wait states around it cover the vector write -> lane permute -> vector
// read sequence, which the compiler cannot see into.
__device__ __forceinline__ float max_with_other_half(float x) {
  float lo = x, hi = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(lo), "+v"(hi));
  return fmaxf(lo, hi);
}

template <int D, bool CAUSAL, bool RESIDENT>
__global__ __launch_bounds__(kThreads, (D == 64 ? 3 : 2)) void exact_bf16_kernel(const ExactArgs a) {
  constexpr int PPR = D / 8;                          // 16-byte pieces per row
  constexpr int NCOPY = kLChunk * PPR / kWave / 4;    // copy instructions per wave, tensor, chunk
  __shared__ __attribute__((aligned(16))) bf16_t kb0[kLChunk * D];
  __shared__ __attribute__((aligned(16))) bf16_t vb0[kLChunk * D];
  __shared__ __attribute__((aligned(16))) bf16_t kb1[kLChunk * D];
  __shared__ __attribute__((aligned(16))) bf16_t vb1[kLChunk * D];
  // wave-private output staging of the resident mode (16 rows x 64 columns per pass)
  __shared__ __attribute__((aligned(16))) bf16_t ost_small[4 * 16 * kOStride];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it scalar
  const int il = lane & 31, kh = lane >> 5;
  const int S = a.S, g = a.Hq / a.Hkv;
  // The scale as a scalar register written by a vector instruction: a register that comes
  // straight from a scalar load makes the compiler wait for "all scalar and LDS traffic" before
  // its first use in a loop iteration, which drains the operand reads in flight.
  const float scale_log2e = __builtin_bit_cast(
      float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, a.scale_log2e) + (lane & 0)));
  // Sequences of up to 128 keys are RESIDENT: both 64-key chunks of K and V sit in the two
  // stages for the whole tile, the workgroup walks all heads_per_wg query heads that share
  // them, and between the one barrier after the copy and the end of the tile the four waves
  // never meet again.  Longer sequences stream chunks through the stages, one head per tile.

  // per tile (the helpers below read these by reference)
  int u = 0, h = 0, R = 0, b = 0, r0 = 0, n_chunk = 0;
  int Sk = S;   // keys this tile's queries may see at all: the sentence's length in a padded batch
  bool active = false;
  const bf16_t* Ksrc = nullptr;
  const bf16_t* Vsrc = nullptr;

  // ---- copies: instruction k = wave + 4 i fills LDS slots [64 k, 64 k + 64), slot = row * PPR +
  // position.  From one instruction to the next, row grows by 256 / PPR (which leaves both
  // permutations unchanged) and both addresses by 2048 elements: one lane offset per tensor.
  const int slot0 = kWave * wave + lane;
  const int crow = slot0 / PPR, cpos = slot0 % PPR;
  const int kpiece = cpos ^ k_piece_swizzle<D>(crow);   // global piece that lands in this lane's slot
  const int vpiece = cpos ^ v_piece_swizzle<D>(crow);
  // Running source pointers, one per tensor, advanced by one chunk after each use (cheaper
  // than rebuilding 64-bit addresses from the chunk index every time).
  const bf16_t* kptr = nullptr;   // set per tile
  const bf16_t* vptr = nullptr;
  auto prefetch = [&](bf16_t* kb, bf16_t* vb, int c) {
    const int nj = min(kLChunk, S - c * kLChunk);
    if (nj == kLChunk) {
#pragma unroll
      for (int i = 0; i < NCOPY; ++i) {
        __builtin_amdgcn_global_load_lds(kptr + 2048 * i, kb + kWave * 8 * (wave + 4 * i), 16, 0, 0);
        __builtin_amdgcn_global_load_lds(vptr + 2048 * i, vb + kWave * 8 * (wave + 4 * i), 16, 0, 0);
      }
      kptr += kLChunk * D;
      vptr += kLChunk * D;
    } else {
      // ragged last chunk: rows past the end repeat the last row (finite, and masked later)
      const bf16_t* ksrc = Ksrc + (size_t)c * kLChunk * D;
      const bf16_t* vsrc = Vsrc + (size_t)c * kLChunk * D;
#pragma unroll
      for (int i = 0; i < NCOPY; ++i) {
        const int rr = min(crow + (256 / PPR) * i, nj - 1);
        __builtin_amdgcn_global_load_lds(ksrc + (size_t)rr * D + 8 * kpiece,
                                         kb + kWave * 8 * (wave + 4 * i), 16, 0, 0);
        __builtin_amdgcn_global_load_lds(vsrc + (size_t)rr * D + 8 * vpiece,
                                         vb + kWave * 8 * (wave + 4 * i), 16, 0, 0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  // ---- operand addresses (elements, relative to a stage; the 32-key block enters as a constant)
  // K operand of column step ks: row il of the block, piece 2 ks + kh
  int koff[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ++ks) koff[ks] = il * D + 8 * ((2 * ks + kh) ^ k_piece_swizzle<D>(il));
  // V^T operand: contraction slot e of lane half kh, step s2, is key 16 s2 + 8 (e / 4) + 4 kh +
  // e % 4 of the block, which is where the first product left the scores in the registers.
  // Lane i of a 16-lane group names key 4 kh + 8 half + i / 4 and the four d from
  // 32 db + 16 (il / 16) + 4 (i % 4).
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
  f32x16 acc[D / 32];
  float m_run = -INFINITY, l_run = 0.f;
  // this wave's 32 query rows of head h as the column operand of the first product, and a
  // fresh accumulator.  (A wave whose rows lie beyond a ragged end works on a copy of the last
  // row and stores nothing: the streaming loop then needs no per-wave branch, whose merge
  // would cost a copy of the accumulator per chunk.)
  auto begin_head = [&]() {
    const bf16_t* qrow = reinterpret_cast<const bf16_t*>(a.Q) +
                         (((size_t)b * a.Hq + h) * S + min(r0 + il, S - 1)) * D + 8 * kh;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) q[ks] = *reinterpret_cast<const u32x4*>(qrow + 16 * ks);
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;
    m_run = -INFINITY;
    l_run = 0.f;
  };

  // ---- pieces of one chunk step (32-key block jb of the stage)
  // scores^T of block jb: 32 keys x 32 query rows, this lane: query row il, 16 of the keys
  auto qk = [&](const bf16_t* kb, int jb) {
    f32x16 s;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks)
      s = mfma_bf16(*reinterpret_cast<const bf16x8*>(kb + koff[ks] + 32 * jb * D),
                    __builtin_bit_cast(bf16x8, q[ks]), s);
    return s;
  };
  // hide the keys this query row must not see (beyond the diagonal or the end of the sentence)
  auto hide = [&](f32x16& s, int c, int jb) {
    const int limit = (CAUSAL ? min(r0 + il, Sk - 1) : Sk - 1) - c * kLChunk - 32 * jb - 4 * kh;
#pragma unroll
    for (int v = 0; v < 16; ++v)
      if (8 * (v >> 2) + (v & 3) > limit) s[v] = -INFINITY;
  };
  // largest score of the query row: in-lane over 16 keys, then across the two lane halves
  auto row_max = [&](const f32x16& s) {
    float m01 = fmaxf(fmaxf(s[0], s[1]), s[2]);
    float m02 = fmaxf(fmaxf(s[3], s[4]), s[5]);
    float m03 = fmaxf(fmaxf(s[6], s[7]), s[8]);
    float m04 = fmaxf(fmaxf(s[9], s[10]), s[11]);
    float m05 = fmaxf(fmaxf(s[12], s[13]), s[14]);
    float mx = fmaxf(fmaxf(fmaxf(m01, m02), m03), fmaxf(fmaxf(m04, m05), s[15]));
    return max_with_other_half(mx);
  };
  // probabilities 2^(score * scale_log2e - m) as the packed bf16 operand of the second product;
  // their sum is taken over the ROUNDED values (the ones that are multiplied with V), two per
  // instruction, so numerator and denominator of the softmax see the same weights
  typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));
  auto probs = [&](const f32x16& s, float m, u32x4 (&pw)[2], float& sum) {
    const bf16x2 ones = {(bf16_t)1.0f, (bf16_t)1.0f};
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float e0 = __builtin_amdgcn_exp2f(fmaf(s[8 * s2 + 2 * w], scale_log2e, -m));
        const float e1 = __builtin_amdgcn_exp2f(fmaf(s[8 * s2 + 2 * w + 1], scale_log2e, -m));
        const uint32_t pk = pack_bf16(e0, e1);
        pw[s2][w] = pk;
        sum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pk), ones, sum, false);
      }
  };
  auto pv = [&](const bf16_t* vb, int jb, const u32x4 (&pw)[2]) {
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int db = 0; db < D / 32; ++db)
        acc[db] = mfma_bf16(vop(vb, db, jb, s2), __builtin_bit_cast(bf16x8, pw[s2]), acc[db]);
  };
  auto rescale = [&](float m_new) {
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
    l_run *= alpha;
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[db][v] *= alpha;
  };

  // One chunk = two 32-key blocks, each with its own online-softmax step, ordered so that
  // matrix and vector work of ONE wave can overlap (the matrix pipe runs asynchronously, but a
  // wave issues in order): the scores of block 1 are requested before the exponentials of
  // block 0 are taken, the second product of block 0 before the exponentials of block 1.
  // The reference point m of a row (weights are 2^(score - m)) follows the row maximum lazily:
  // it moves, and the accumulator is rescaled, only when some row of the wave has outgrown
  // its reference by more than kRescaleSlack, so weights stay below 2^kRescaleSlack and almost
  // every step skips the rescaling (a new maximum turns up in nearly every block of random
  // scores, a jump by 2^8 hardly ever); the final division by the row sum makes the result
  // independent of m.  For block 1 the rescaling happens after the second product of block 0
  // has been added (those weights refer to the old m).
  // MASKED is the variant for chunks that touch the diagonal or the ragged end (nblk of the
  // two blocks exist for this wave, some of their keys may be hidden); the other variant has no
  // per-element tests.  The flag is a literal at every call site and the body is inlined.
  auto step = [&](const bf16_t* kb, const bf16_t* vb, int c, int nblk, const bool MASKED)
      __attribute__((always_inline)) {
    const bool two = !MASKED || nblk > 1;
    f32x16 s0 = qk(kb, 0);
    if (MASKED) hide(s0, c, 0);
    float m0 = m_run;
    {
      const float cand = fmaxf(m_run, row_max(s0) * scale_log2e);
      if (__any(cand > m_run + kRescaleSlack)) {
        rescale(cand);
        m0 = cand;
      }
    }
    m_run = m0;
    f32x16 s1;
    if (two) s1 = qk(kb, 1);
    u32x4 p0[2];
    float sum0 = 0.f;
    probs(s0, m0, p0, sum0);
    l_run += sum0;
    if (two) {
      if (MASKED) hide(s1, c, 1);
      const float cand1 = fmaxf(m0, row_max(s1) * scale_log2e);
      const bool moved = __any(cand1 > m0 + kRescaleSlack);
      const float m1 = moved ? cand1 : m0;
      pv(vb, 0, p0);
      u32x4 p1[2];
      float sum1 = 0.f;
      probs(s1, m1, p1, sum1);
      if (moved) rescale(m1);
      m_run = m1;
      l_run += sum1;
      pv(vb, 1, p1);
    } else {
      pv(vb, 0, p0);
    }
  };
  // chunk c through the masked variant (exact for every chunk, only slower)
  auto tail_step = [&](const bf16_t* kb, const bf16_t* vb, int c) {
    if (!active) return;
    const int nj = min(kLChunk, Sk - c * kLChunk);
    int nblk = (nj + 31) >> 5;
    if (CAUSAL) nblk = min(nblk, (r0 >> 5) + 1 - 2 * c);
    if (nblk > 0) step(kb, vb, c, nblk, true);
  };
  // this wave's copies have landed (they are counted like loads), then everybody's; the
  // barrier also retires the stage that the next copy overwrites
  auto publish = [&]() {
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
  };

  // the 32 x D result of this wave in 16 x 64 passes through its small private buffer (the
  // stages still hold K and V for the next head); every global store covers whole 128-byte lines
  auto store_small = [&](bf16_t* Oh, float inv) {
    bf16_t* ost = ost_small + wave * (16 * kOStride);
#pragma unroll
    for (int rh = 0; rh < 2; ++rh)
#pragma unroll
      for (int dh = 0; dh < D / 64; ++dh) {
        if ((il >> 4) == rh) {
#pragma unroll
          for (int dbp = 0; dbp < 2; ++dbp)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
              const f32x16& t = acc[2 * dh + dbp];
              u32x2 w;
              w.x = pack_bf16(t[4 * vq] * inv, t[4 * vq + 1] * inv);
              w.y = pack_bf16(t[4 * vq + 2] * inv, t[4 * vq + 3] * inv);
              *reinterpret_cast<u32x2*>(ost + (il & 15) * kOStride + 32 * dbp + 8 * vq + 4 * kh) = w;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int it = 0; it < 2; ++it) {
          const int p = it * kWave + lane;
          const int row = p >> 3, c8 = p & 7;
          const u32x2* sp = reinterpret_cast<const u32x2*>(ost + row * kOStride + 8 * c8);
          u32x2 lo = sp[0], hi = sp[1];
          __builtin_nontemporal_store(
              u32x4{lo.x, lo.y, hi.x, hi.y},
              reinterpret_cast<u32x4*>(Oh + (size_t)(16 * rh + row) * D + 64 * dh + 8 * c8));
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
  };

  if constexpr (RESIDENT) {
    // A fixed number of workgroups, each taking every gridDim.x-th tile: the copies of the next
    // tile's K and V are started before the last head of the current tile is written out, so
    // stores and loads of one workgroup overlap, and a tile whose batch item was served by the
    // reuse branch costs no workgroup launch.  Which of its tiles have work a workgroup finds
    // out 64 candidates at a time: lane i tests candidate i (one vector load of the routing
    // flags, one round trip to memory for all of them) and the votes form a wave-uniform bit
    // mask that the walk below consumes with scalar bit operations.
    const int hslots = g / a.heads_per_wg;
    int cand_base = 0;          // candidates cand_base .. cand_base + 63 are in `live`
    unsigned long long live = 0;
    auto scan = [&](int base) {
      // (tile numbers stay below 2^31 + 64 gridDim.x: unsigned 32-bit arithmetic is enough)
      const unsigned t = blockIdx.x + (unsigned)(base + lane) * gridDim.x;
      bool work = false;
      if (t < (unsigned)a.n_blocks) {
        const int ti = (int)t;
        const int ut = ((ti >> 3) / hslots) * 8 + (ti & 7);   // ids equal mod 8 (one XCD) share K, V
        work = ut < a.n_kvtiles && !(a.row_sel && a.row_sel[ut / a.Hkv] >= 0);
      }
      cand_base = base;
      live = __ballot(work);
    };
    // first tile with work among this workgroup's candidates number `from` and up, or -1
    auto locate = [&](int from) {
      while (true) {
        const int shift = from - cand_base;
        const unsigned long long rest = shift < 64 ? (live >> shift) : 0ull;
        if (rest) {
          const int i = from + __builtin_ctzll(rest);
          return (int)(blockIdx.x + (unsigned)i * gridDim.x);
        }
        const int next = cand_base + 64;
        if (blockIdx.x + (unsigned)next * gridDim.x >= (unsigned)a.n_blocks) return -1;
        scan(next);
        from = next;
      }
    };
    scan(0);
    int h_first = 0;
    auto enter = [&](int t) {       // tile variables, and its K and V on their way
      const int slot = t >> 3;
      u = (slot / hslots) * 8 + (t & 7);
      h_first = (u % a.Hkv) * g + (slot % hslots) * a.heads_per_wg;
      b = u / a.Hkv;
      Ksrc = reinterpret_cast<const bf16_t*>(a.K) + (size_t)u * S * D;
      Vsrc = reinterpret_cast<const bf16_t*>(a.V) + (size_t)u * S * D;
      kptr = Ksrc + crow * D + 8 * kpiece;
      vptr = Vsrc + crow * D + 8 * vpiece;
      Sk = a.key_len ? min(max(a.key_len[b], 1), S) : S;
      n_chunk = (Sk + kLChunk - 1) / kLChunk;
      prefetch(kb0, vb0, 0);
      if (n_chunk > 1) prefetch(kb1, vb1, 1);
    };
    int t = locate(0);
    if (t < 0) return;   // e.g. a batch served entirely by the reuse branch
    enter(t);
    while (true) {
      publish();
      const int rot = (t >> 3) & 3;
      for (int hl = 0; hl < a.heads_per_wg; ++hl) {
        h = h_first + hl;
        // causal work grows with the row block and wave i always runs on SIMD i: rotating the
        // wave -> row block assignment lets every SIMD see the same mix
        r0 = 32 * ((wave + rot + hl) & 3);
        active = r0 < S;
        begin_head();
        for (int c = 0; c < n_chunk; ++c) tail_step(c ? kb1 : kb0, c ? vb1 : vb0, c);
        if (hl + 1 == a.heads_per_wg) break;   // the last head is written after the next copies start
        if (active) {
          const float inv = 1.0f / (l_run + __shfl_xor(l_run, 32));
          store_small(reinterpret_cast<bf16_t*>(a.O) + (((size_t)b * a.Hq + h) * S + r0) * (size_t)D, inv);
        }
      }
      const float inv = 1.0f / (l_run + __shfl_xor(l_run, 32));
      bf16_t* Olast = reinterpret_cast<bf16_t*>(a.O) + (((size_t)b * a.Hq + h) * S + r0) * (size_t)D;
      const bool act = active;
      const int tn = locate((t - (int)blockIdx.x) / (int)gridDim.x + 1);
      __syncthreads();          // every wave has finished reading the stages
      if (tn >= 0) enter(tn);
      if (act) store_small(Olast, inv);   // registers and the wave's own small buffer only
      if (tn < 0) break;
      t = tn;
    }
  } else {
    // one tile per workgroup: (K/V tile u, head, row block R), heaviest row blocks first
    const int bid = blockIdx.x;
    const int slot = bid >> 3;
    const int per_u = g * a.n_rblk;
    u = (slot / per_u) * 8 + (bid & 7);   // ids equal mod 8 (one XCD) share K, V in its L2
    if (u >= a.n_kvtiles) return;
    h = (u % a.Hkv) * g + (slot % per_u) / a.n_rblk;
    R = a.n_rblk - 1 - (slot % per_u) % a.n_rblk;
    b = u / a.Hkv;
    if (a.row_sel && a.row_sel[b] >= 0) return;
    Ksrc = reinterpret_cast<const bf16_t*>(a.K) + (size_t)u * S * D;
    Vsrc = reinterpret_cast<const bf16_t*>(a.V) + (size_t)u * S * D;
    kptr = Ksrc + crow * D + 8 * kpiece;
    vptr = Vsrc + crow * D + 8 * vpiece;
    Sk = a.key_len ? min(max(a.key_len[b], 1), S) : S;
    const int last_key = CAUSAL ? min(Sk, kChunk * (R + 1)) : Sk;
    n_chunk = (last_key + kLChunk - 1) / kLChunk;
    r0 = R * kChunk + 32 * wave;
    active = r0 < S;
    begin_head();
    // Chunks below c_split are complete and fully visible to every wave of the workgroup
    // (they lie left of the diagonal blocks of all 128 rows, and before a ragged end): the
    // main loop runs only the test-free variant, two chunks per trip so that stages
    // alternate without pointer arithmetic.  The few chunks from c_split on go through the
    // masked variant.
    const int c_split = CAUSAL ? min(2 * R, Sk / kLChunk) : Sk / kLChunk;
    prefetch(kb0, vb0, 0);
    int c = 0;
    for (; c + 1 < c_split; c += 2) {
      publish();
      prefetch(kb1, vb1, c + 1);
      step(kb0, vb0, c, 2, false);
      publish();
      if (c + 2 < n_chunk) prefetch(kb0, vb0, c + 2);
      step(kb1, vb1, c + 1, 2, false);
    }
    // (one copy of the masked code: the stage is picked at run time, which only costs the
    // compiler its proof that copy and reads touch different arrays, i.e. some overlap)
    for (; c < n_chunk; ++c) {
      publish();
      bf16_t* kcur = (c & 1) ? kb1 : kb0;
      bf16_t* vcur = (c & 1) ? vb1 : vb0;
      if (c + 1 < n_chunk) prefetch((c & 1) ? kb0 : kb1, (c & 1) ? vb0 : vb1, c + 1);
      tail_step(kcur, vcur, c);
    }
    __syncthreads();   // every wave is done with both stages: they now stage the output
    if (active) {
      const float inv = 1.0f / (l_run + __shfl_xor(l_run, 32));
      bf16_t* Oh = reinterpret_cast<bf16_t*>(a.O) + (((size_t)b * a.Hq + h) * S + r0) * (size_t)D;
      bf16_t* ost = wave == 0 ? kb0 : wave == 1 ? vb0 : wave == 2 ? kb1 : vb1;
      store_tile_bf16<D>(acc, inv, ost, Oh, lane);
    }
  }
}

// fp32 path (vector ALUs): one wave per (batch item, head, query row).
__global__ __launch_bounds__(kWave) void exact_f32_kernel(const ExactArgs a, int D, int causal,
                                                          float scale) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* p = reinterpret_cast<float*>(smem);   // [S]
  const int S = a.S, g = a.Hq / a.Hkv;
  const int i = blockIdx.x % S;
  const int h = (blockIdx.x / S) % a.Hq;
  const int b = blockIdx.x / (S * a.Hq);
  if (a.row_sel && a.row_sel[b] >= 0) return;
  const int lane = threadIdx.x;
  const float* q = reinterpret_cast<const float*>(a.Q) + (((size_t)b * a.Hq + h) * S + i) * (size_t)D;
  const float* K = reinterpret_cast<const float*>(a.K) + ((size_t)b * a.Hkv + h / g) * (size_t)S * D;
  const float* V = reinterpret_cast<const float*>(a.V) + ((size_t)b * a.Hkv + h / g) * (size_t)S * D;
  float* o = reinterpret_cast<float*>(a.O) + (((size_t)b * a.Hq + h) * S + i) * (size_t)D;
  const int len = a.key_len ? min(max(a.key_len[b], 1), S) : S;   // keys beyond it are padding
  const int nj = min(causal ? i + 1 : S, len);
  float mx = -INFINITY;
  for (int j = lane; j < nj; j += kWave) {
    float acc = 0.f;
    for (int d = 0; d < D; ++d) acc = fmaf(q[d], K[(size_t)j * D + d], acc);
    acc *= scale;
    p[j] = acc;
    mx = fmaxf(mx, acc);
  }
  for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  float z = 0.f;
  for (int j = lane; j < nj; j += kWave) {
    const float e = expf(p[j] - mx);
    p[j] = e;
    z += e;
  }
  for (int off = 32; off > 0; off >>= 1) z += __shfl_xor(z, off);
  __syncthreads();
  for (int d = lane; d < D; d += kWave) {
    float acc = 0.f;
    for (int j = 0; j < nj; ++j) acc = fmaf(p[j], V[(size_t)j * D + d], acc);
    o[d] = acc / z;
  }
}

template <int D, bool CAUSAL, bool RESIDENT>
static hipError_t launch_exact_bf16_r(ExactArgs a, dim3 grid, hipStream_t stream) {
  a.n_blocks = (int32_t)grid.x;
  // resident launch: at most 32 workgroups per compute unit walk the tiles (enough of them for
  // the hardware to even out an uneven mix of hits and misses -- fewer, longer-lived workgroups
  // measured 2-5 % slower; a multiple of 8 keeps a workgroup's tiles on its own XCD)
  // The resident variant walks its tiles with a fixed number of workgroups.  Dispatching a
  // workgroup takes time even when it finds nothing to do (some 420 workgroups start per
  // microsecond: 8,192 of them cost the 19 us that a launch on a batch without misses used to
  // take), so a routed launch, which may find little or nothing, gets half as many.  Fewer
  // still would help that case more (2,048: 7 instead of 9 us) but costs a launch with many
  // misses its load balance (64 of 128 items at the 8B shape: 4-9 % slower, the hardware
  // balances many short-lived workgroups better than few long-lived ones); 4,096 costs nothing
  // measurable there.
  if (RESIDENT) {
    const unsigned cap = a.row_sel ? 4096u : 8192u;
    if (grid.x > cap) grid.x = cap;
  }
  hipLaunchKernelGGL((exact_bf16_kernel<D, CAUSAL, RESIDENT>), grid, dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

template <int D, bool CAUSAL>
static hipError_t launch_exact_bf16(const ExactArgs& a, dim3 grid, hipStream_t stream) {
  return a.n_rblk == 1 ? launch_exact_bf16_r<D, CAUSAL, true>(a, grid, stream)
                       : launch_exact_bf16_r<D, CAUSAL, false>(a, grid, stream);
}

hipError_t launch_exact(const ExactLaunch& p, hipStream_t stream) {
  if (p.B == 0) return hipSuccess;
  ExactArgs a;
  a.Q = p.Q; a.K = p.K; a.V = p.V; a.O = p.O; a.row_sel = p.row_sel; a.key_len = p.key_len;
  a.B = p.B; a.Hq = p.Hq; a.Hkv = p.Hkv; a.S = p.S;
  a.n_rblk = (p.S + kChunk - 1) / kChunk;
  a.n_kvtiles = p.B * p.Hkv;
  const float scale = p.scale == 0.f ? 1.0f / sqrtf((float)p.D) : p.scale;
  a.scale_log2e = scale * 1.44269504088896340736f;
  a.heads_per_wg = 1;
  if (p.is_f32) {
    const unsigned blocks = (unsigned)((size_t)p.B * p.Hq * p.S);
    hipLaunchKernelGGL(exact_f32_kernel, dim3(blocks), dim3(kWave), (size_t)p.S * sizeof(float),
                       stream, a, p.D, p.causal, scale);
    return hipGetLastError();
  }
  const int g = p.Hq / p.Hkv;
  a.heads_per_wg = a.n_rblk == 1 ? g : 1;
  const int u8 = (a.n_kvtiles + 7) / 8 * 8;
  const dim3 grid((unsigned)((size_t)u8 * (g / a.heads_per_wg) * a.n_rblk));
  if (p.D == 64)
    return p.causal ? launch_exact_bf16<64, true>(a, grid, stream)
                    : launch_exact_bf16<64, false>(a, grid, stream);
  return p.causal ? launch_exact_bf16<128, true>(a, grid, stream)
                  : launch_exact_bf16<128, false>(a, grid, stream);
}

}  // namespace ac
