// Algorithm 1, search and threshold steps: exact top-k similarity search of a
// batch of query feature vectors against the whole feature-vector database,
// then hit / miss routing.  (The paper uses an approximate graph index; this
// is the exact search that index approximates.)
//
// Two phases.
//  1. score + group maximum.  The database rows are split into contiguous
//     groups (one workgroup each).  The N x B score matrix is never written:
//     a workgroup forms its scores on the matrix cores (fp16 inputs, fp32
//     accumulation) and keeps, per query, only the best (score, row) of the
//     group under the order "higher score, then lower row".
//  2. finalise.  k = 1: the best group maximum is the answer.  k > 1: every
//     member of the exact top-k lies in one of the k groups with the best
//     maxima (each such group holds at least one of the k best elements), so
//     those k groups are re-scored row by row and the k best rows selected.
// fp32 databases (and the L2 metric) use a vector-ALU phase 1 of the same shape.
#include "common.hpp"
#include "launch.hpp"

namespace ac {

constexpr int kQPad = 8;            // fp16 elements of padding per staged query row
constexpr int kValuRowsPerWg = 256;
constexpr int kIdxNone = 0x7fffffff;

struct SearchArgs {
  const void* emb;
  const void* q;
  const int32_t* map_of;
  int32_t N, E, B, k, metric;
  int32_t q0, nq;          // query super-block handled by this launch (phase 1)
  int32_t rows_per_wg, G;  // group size and count (a group: the rows one partial result covers)
  int32_t wg_rows;         // rows one phase-1 workgroup scans: the group, or four groups of 32
  float threshold;
  float* part_s;           // [B][G]
  int32_t* part_i;         // [B][G]
  float* cand;             // [B][k * rows_per_wg] (k > 1 only)
  int32_t* idx;
  float* score;
  int32_t* hit;
};

// (s1, i1) ranks before (s0, i0): higher score, or equal score and lower row.
__device__ __forceinline__ bool ranks_before(float s1, int i1, float s0, int i0) {
  return s1 > s0 || (s1 == s0 && i1 < i0);
}

// Best (score, row) over a workgroup; result valid in every thread.
__device__ __forceinline__ void block_argmax(float& s, int& i, float* red_s, int* red_i) {
  for (int off = 32; off > 0; off >>= 1) {
    const float so = __shfl_xor(s, off);
    const int io = __shfl_xor(i, off);
    if (ranks_before(so, io, s, i)) { s = so; i = io; }
  }
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();   // red_* may still be read from a previous call
  if ((threadIdx.x & 63) == 0) { red_s[wave] = s; red_i[wave] = i; }
  __syncthreads();
  s = red_s[0]; i = red_i[0];
  for (int w = 1; w < nw; ++w)
    if (ranks_before(red_s[w], red_i[w], s, i)) { s = red_s[w]; i = red_i[w]; }
}

// ---------------------------------------------------------------- phase 1, matrix cores
template <int KSMAX, int NQB>
__global__ __launch_bounds__(kThreads) void search_f16_kernel(const SearchArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int E = a.E, QS = E + kQPad;
  f16_t* qs = reinterpret_cast<f16_t*>(smem);                                 // [32 NQB][QS]
  float* red_s = reinterpret_cast<float*>(smem + (size_t)32 * NQB * QS * 2);  // [4][32 NQB]
  int* red_i = reinterpret_cast<int*>(red_s + 4 * 32 * NQB);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it scalar
  const int il = lane & 31, kh = lane >> 5;
  const int nks = E >> 4;

  // stage the query super-block, zero rows beyond nq
  {
    const int EQ = E >> 3;
    const u32x4* src = reinterpret_cast<const u32x4*>(reinterpret_cast<const f16_t*>(a.q) +
                                                      (size_t)a.q0 * E);
    for (int p = tid; p < 32 * NQB * EQ; p += kThreads) {
      const int r = p / EQ, c = p % EQ;
      u32x4 w = {0u, 0u, 0u, 0u};
      if (r < a.nq) w = src[(size_t)r * EQ + c];
      *reinterpret_cast<u32x4*>(qs + r * QS + 8 * c) = w;
    }
  }
  __syncthreads();

  float best_s[NQB];
  int best_i[NQB];
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) { best_s[qb] = -INFINITY; best_i[qb] = kIdxNone; }

  const int row_begin = blockIdx.x * a.wg_rows;
  const int row_end = min(row_begin + a.wg_rows, a.N);
  const f16_t* emb = reinterpret_cast<const f16_t*>(a.emb);
  for (int rb = row_begin + 32 * wave; rb < row_end; rb += 128) {
    // database operand: lane (il, kh) holds emb[rb + il][16 ks + 8 kh .. +8); rows past the
    // end are clamped for the load and masked below
    const int rowc = min(rb + il, a.N - 1);
    const f16_t* erow = emb + (size_t)rowc * E + 8 * kh;
    f16x8 e[KSMAX];
#pragma unroll
    for (int ks = 0; ks < KSMAX; ++ks)
      if (ks < nks) e[ks] = *reinterpret_cast<const f16x8*>(erow + 16 * ks);
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
      f32x16 acc;
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = 0.f;
      const f16_t* qrow = qs + (32 * qb + il) * QS + 8 * kh;
#pragma unroll
      for (int ks = 0; ks < KSMAX; ++ks)
        if (ks < nks) acc = mfma_f16(e[ks], *reinterpret_cast<const f16x8*>(qrow + 16 * ks), acc);
      // acc[v] = <emb[rb + mfma_row(v)], q[32 qb + il]>; rows ascend with v, so a strict
      // comparison keeps the lowest row among equal scores
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = rb + mfma_row(v, kh);
        const float s = r < a.N ? acc[v] : -INFINITY;
        if (s > best_s[qb]) { best_s[qb] = s; best_i[qb] = r; }
      }
    }
  }
  // combine the two lane halves
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    const float so = __shfl_xor(best_s[qb], 32);
    const int io = __shfl_xor(best_i[qb], 32);
    if (ranks_before(so, io, best_s[qb], best_i[qb])) { best_s[qb] = so; best_i[qb] = io; }
  }
  if (a.rows_per_wg == 32) {
    // groups of 32 rows (top-k searches: the finalising kernel re-scores k whole groups per
    // query, so small groups are cheap): a workgroup scans 128 rows in one pass and every
    // wave's 32 rows are a group of their own -- nothing to merge
    const int gi = 4 * blockIdx.x + wave;
    if (kh == 0 && gi < a.G) {
#pragma unroll
      for (int qb = 0; qb < NQB; ++qb) {
        const int t = 32 * qb + il;
        if (t < a.nq) {
          a.part_s[(size_t)(a.q0 + t) * a.G + gi] = best_s[qb];
          a.part_i[(size_t)(a.q0 + t) * a.G + gi] = best_i[qb];
        }
      }
    }
    return;
  }
  // one group per workgroup: the four waves meet in LDS
#pragma unroll
  for (int qb = 0; qb < NQB; ++qb) {
    if (kh == 0) {
      red_s[wave * 32 * NQB + 32 * qb + il] = best_s[qb];
      red_i[wave * 32 * NQB + 32 * qb + il] = best_i[qb];
    }
  }
  __syncthreads();
  for (int t = tid; t < a.nq; t += kThreads) {
    float s = red_s[t];
    int i = red_i[t];
    for (int w = 1; w < 4; ++w) {
      const float so = red_s[w * 32 * NQB + t];
      const int io = red_i[w * 32 * NQB + t];
      if (ranks_before(so, io, s, i)) { s = so; i = io; }
    }
    a.part_s[(size_t)(a.q0 + t) * a.G + blockIdx.x] = s;
    a.part_i[(size_t)(a.q0 + t) * a.G + blockIdx.x] = i;
  }
}

// ---------------------------------------------------------------- phase 1, query-stationary
// For more than 64 queries, and for large databases at any batch size, the roles are swapped: the QUERIES live in registers (each of the
// four waves keeps QPW blocks of 32 queries as MFMA column operands for the whole kernel) and
// the database rows stream through LDS in chunks of 64 rows.  Every row operand read from LDS
// feeds QPW MFMAs per wave and is shared by the four waves, so LDS traffic is 4x the HBM
// stream instead of 32x, and no cross-wave reduction is needed (a wave owns its queries).
//
// The chunks are copied global -> LDS directly (global_load_lds_dwordx4: no data registers; a
// wave instruction fills 1 KiB of LDS contiguously, lane l at base + 16 l, whatever global
// address lane l names), double-buffered in two separate LDS arrays so that the copy of chunk
// c+1 runs while chunk c is multiplied.  Rows are stored unpadded; piece p (16 bytes) of row r
// sits at position p ^ (r & 15) of its row, which makes the 16-byte operand reads of 32
// consecutive rows conflict-free; the copy obtains the swizzle for free by choosing which
// global piece each lane fetches.
constexpr int kBigRows = 64;   // database rows per LDS chunk

template <int KSMAX, int QPW>
__global__ __launch_bounds__(kThreads, (KSMAX == 32 ? 1 : 2)) void search_f16_big_kernel(const SearchArgs a) {
  constexpr int E = 16 * KSMAX;               // this kernel is built for E = 128, 256, 512
  constexpr int EQ = E / 8;                   // 16-byte pieces per row
  constexpr int NDMA = kBigRows * EQ / kWave / 4;   // copy instructions per wave and chunk
  __shared__ __attribute__((aligned(16))) f16_t buf0[kBigRows * E];
  __shared__ __attribute__((aligned(16))) f16_t buf1[kBigRows * E];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it scalar
  const int il = lane & 31, kh = lane >> 5;

  // query operands: lane (il, kh) keeps q[q0 + 32 (QPW wave + j) + il][16 ks + 8 kh .. +8)
  f16x8 qop[QPW][KSMAX];
#pragma unroll
  for (int j = 0; j < QPW; ++j) {
    const int qi = 32 * (QPW * wave + j) + il;
    const f16_t* qrow = reinterpret_cast<const f16_t*>(a.q) + (size_t)(a.q0 + min(qi, a.nq - 1)) * E + 8 * kh;
#pragma unroll
    for (int ks = 0; ks < KSMAX; ++ks) {
      qop[j][ks] = *reinterpret_cast<const f16x8*>(qrow + 16 * ks);
      if (qi >= a.nq) {   // padding query: all-zero operand
#pragma unroll
        for (int e = 0; e < 8; ++e) qop[j][ks][e] = (f16_t)0.f;
      }
    }
  }

  const int row_begin = blockIdx.x * a.rows_per_wg;
  const int row_end = min(row_begin + a.rows_per_wg, a.N);
  const int n_chunk = (row_end - row_begin + kBigRows - 1) / kBigRows;
  const f16_t* emb = reinterpret_cast<const f16_t*>(a.emb);

  // copy chunk ch into buf: instruction k = wave + 4 i fills LDS slots [64 k, 64 k + 64) of the
  // chunk (slot = row * EQ + position).  The element offset of the global piece a lane fetches
  // with instruction i, relative to the chunk's first row, is fixed for the whole kernel.
  unsigned coff[NDMA];
#pragma unroll
  for (int i = 0; i < NDMA; ++i) {
    const int slot = kWave * (wave + 4 * i) + lane;
    const int row = slot / EQ, pos = slot % EQ;
    coff[i] = (unsigned)(row * E + 8 * (pos ^ (row & 15)));
  }
  auto copy_in = [&](f16_t* buf, int ch) {
    const f16_t* src = emb + (size_t)(row_begin + ch * kBigRows) * E;
#pragma unroll
    for (int i = 0; i < NDMA; ++i) {
      const f16_t* piece = src + coff[i];
      __builtin_amdgcn_global_load_lds(piece, buf + kWave * (wave + 4 * i) * 8, 16, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  // the same for a chunk that reaches beyond the database: rows past the end repeat the last
  // row (they are masked when compared)
  auto copy_in_clamped = [&](f16_t* buf, int ch) {
    const int first = row_begin + ch * kBigRows;
    const f16_t* src = emb + (size_t)first * E;   // uniform; lanes add a small 32-bit offset
    const int last = a.N - 1 - first;
#pragma unroll
    for (int i = 0; i < NDMA; ++i) {
      const int slot = kWave * (wave + 4 * i) + lane;
      const int row = slot / EQ, pos = slot % EQ;
      const unsigned off = (unsigned)(min(row, last) * E + 8 * (pos ^ (row & 15)));
      const f16_t* piece = src + off;
      __builtin_amdgcn_global_load_lds(piece, buf + kWave * (wave + 4 * i) * 8, 16, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  float best_s[QPW];
  int best_i[QPW];
#pragma unroll
  for (int j = 0; j < QPW; ++j) { best_s[j] = -INFINITY; best_i[j] = kIdxNone; }

  // RAGGED is a literal at both call sites and the body is inlined: the copy used for complete
  // chunks carries no per-row tests
  // LDS element offset of this lane's operand piece of contraction step ks (row il of a 32-row
  // block; piece 2 ks + kh at position (2 ks + kh) ^ (il & 15)).  The exchange only touches the
  // low four bits of the piece index, so steps ks and ks + 8 lie exactly 16 pieces apart:
  // eight offsets serve every width, the rest is an immediate.
  int eoff[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) eoff[ks] = il * E + 8 * ((2 * ks + kh) ^ (il & 15));
  auto operand = [&](const f16_t* buf, int rb, int ks) {
    return *reinterpret_cast<const f16x8*>(buf + eoff[ks & 7] + 128 * (ks >> 3) + 32 * rb * E);
  };

  // RAGGED is a literal at both call sites and the body is inlined: the copy used for complete
  // chunks carries no per-row tests.  The operand reads run two steps ahead of the products
  // (three operand registers in rotation), the fences keep that order in the instruction stream.
  auto compute = [&](const f16_t* buf, int ch, const bool RAGGED) __attribute__((always_inline)) {
    const int cbase = row_begin + ch * kBigRows;
    constexpr int NRB = kBigRows / 32;
    f16x8 eop[3];
    eop[0] = operand(buf, 0, 0);
    eop[1] = operand(buf, 0, 1);
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
      f32x16 acc[QPW];
#pragma unroll
      for (int j = 0; j < QPW; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KSMAX; ++ks) {
        const int t = rb * KSMAX + ks;   // step within the chunk: the reads run on into the next block
        if (ks + 2 < KSMAX) eop[(t + 2) % 3] = operand(buf, rb, ks + 2);
        else if (rb + 1 < NRB) eop[(t + 2) % 3] = operand(buf, rb + 1, ks + 2 - KSMAX);
#pragma unroll
        for (int j = 0; j < QPW; ++j) acc[j] = mfma_f16(eop[t % 3], qop[j][ks], acc[j]);
        __builtin_amdgcn_sched_barrier(0);
      }
      // acc[j][v] = <emb[r], q>.  A new best becomes rare as the scan proceeds, so first only the
      // block maximum is compared; the position is looked up only when some lane improved.
      // Rows ascend with v, rb and ch, so strict comparisons keep the lowest row among equals.
      if (RAGGED) {
        const int rbase = cbase + 32 * rb + 4 * kh;
#pragma unroll
        for (int j = 0; j < QPW; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (rbase + 8 * (v >> 2) + (v & 3) >= row_end) acc[j][v] = -INFINITY;
      }
      // Only WHICH 32-row block holds a lane's best score is remembered (one compare and two
      // selects per block and query block); the row inside that block is found by the
      // finalising kernel, which re-scores the 32 rows of the one winning block per query.
      // Looking the position up here was the expensive part: with 64 lanes and a few dozen
      // blocks per workgroup some lane improves in nearly every block, so a wave-wide
      // "did anyone improve" test almost never skipped the 48-instruction search.
      // Blocks ascend with rb and ch, so the strict comparison keeps the lowest block among equals.
      const int blk = ch * (kBigRows / 32) + rb;
#pragma unroll
      for (int j = 0; j < QPW; ++j) {
        float mx = fmaxf(fmaxf(acc[j][0], acc[j][1]), acc[j][2]);
#pragma unroll
        for (int v = 3; v < 15; v += 2) mx = fmaxf(fmaxf(mx, acc[j][v]), acc[j][v + 1]);
        mx = fmaxf(mx, acc[j][15]);
        const bool up = mx > best_s[j];
        best_s[j] = up ? mx : best_s[j];
        best_i[j] = up ? blk : best_i[j];
      }
      // the next block's products must not start before these comparisons are done: a second
      // live set of result registers does not fit next to the query operands
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // own copies landed (they are counted like loads), then everybody's
  auto publish = [&]() {
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
  };

  // Complete chunks run through the test-free copy of the loop body, two per trip so that the
  // buffers alternate without pointer arithmetic; a last incomplete chunk (end of the group
  // or of the database) goes through the clamped copy and the masked comparison.
  const int n_full = (row_end - row_begin) / kBigRows;
  if (n_full > 0) copy_in(buf0, 0); else copy_in_clamped(buf0, 0);
  publish();
  int ch = 0;
  for (; ch + 1 < n_full; ch += 2) {
    copy_in(buf1, ch + 1);
    compute(buf0, ch, false);
    publish();
    if (ch + 2 < n_full) copy_in(buf0, ch + 2);
    else if (ch + 2 < n_chunk) copy_in_clamped(buf0, ch + 2);
    compute(buf1, ch + 1, false);
    publish();
  }
  for (; ch < n_chunk; ++ch) {   // at most one complete and one incomplete chunk are left
    f16_t* cur = (ch & 1) ? buf1 : buf0;
    f16_t* nxt = (ch & 1) ? buf0 : buf1;
    if (ch + 1 < n_chunk) {
      if (ch + 1 < n_full) copy_in(nxt, ch + 1); else copy_in_clamped(nxt, ch + 1);
    }
    compute(cur, ch, true);
    publish();
  }
  // combine the two lane halves; every wave owns its queries, nothing else to merge
#pragma unroll
  for (int j = 0; j < QPW; ++j) {
    if (best_i[j] != kIdxNone)   // block -> its first database row (the stand-in for "the row")
      best_i[j] = row_begin + 32 * best_i[j];
    const float so = __shfl_xor(best_s[j], 32);
    const int io = __shfl_xor(best_i[j], 32);
    if (ranks_before(so, io, best_s[j], best_i[j])) { best_s[j] = so; best_i[j] = io; }
    const int qi = 32 * (QPW * wave + j) + il;
    if (kh == 0 && qi < a.nq) {
      a.part_s[(size_t)(a.q0 + qi) * a.G + blockIdx.x] = best_s[j];
      a.part_i[(size_t)(a.q0 + qi) * a.G + blockIdx.x] = best_i[j];
    }
  }
}

// ------------------------------------------------------------- vector-ALU scoring
template <typename T>
__device__ __forceinline__ float load_as_float(const T* p) { return (float)(*p); }

// score of one database row against the query staged in LDS as fp32
template <typename T>
__device__ __forceinline__ float row_score(const T* __restrict__ row, const float* __restrict__ qf,
                                           int E, int metric) {
  float acc = 0.f;
  if (metric == 0) {
    for (int e = 0; e < E; ++e) acc = fmaf(qf[e], load_as_float(row + e), acc);
  } else {
    for (int e = 0; e < E; ++e) {
      const float d = qf[e] - load_as_float(row + e);
      acc = fmaf(-d, d, acc);
    }
  }
  return acc;
}

// phase 1 on the vector ALUs: grid (G, B); one thread per database row.
template <typename T>
__global__ __launch_bounds__(kThreads) void search_valu_kernel(const SearchArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* qf = reinterpret_cast<float*>(smem);   // [E]
  __shared__ float red_s[4];
  __shared__ int red_i[4];
  const int b = blockIdx.y, gidx = blockIdx.x;
  const T* q = reinterpret_cast<const T*>(a.q) + (size_t)b * a.E;
  for (int e = threadIdx.x; e < a.E; e += kThreads) qf[e] = load_as_float(q + e);
  __syncthreads();
  const int r = gidx * a.rows_per_wg + threadIdx.x;
  float s = -INFINITY;
  int i = kIdxNone;
  if ((int)threadIdx.x < a.rows_per_wg && r < a.N) {
    s = row_score(reinterpret_cast<const T*>(a.emb) + (size_t)r * a.E, qf, a.E, a.metric);
    i = r;
  }
  block_argmax(s, i, red_s, red_i);
  if (threadIdx.x == 0) {
    a.part_s[(size_t)b * a.G + gidx] = s;
    a.part_i[(size_t)b * a.G + gidx] = i;
  }
}

// ------------------------------------------------------------------- phase 2
__device__ __forceinline__ void write_hit(const SearchArgs& a, int b, float s0, int i0) {
  if (i0 == kIdxNone) {   // no row ranked at all (every score of the query is NaN): a miss
    a.hit[b] = -1;
    return;
  }
  float sim = s0;
  if (a.metric == 1) sim = 1.0f - sqrtf(-s0);
  int entry = a.map_of ? a.map_of[i0] : i0;
  a.hit[b] = (sim >= a.threshold) ? entry : -1;
}

// k = 1: best of the group maxima.
__global__ __launch_bounds__(kThreads) void finalize_top1_kernel(const SearchArgs a) {
  __shared__ float red_s[4];
  __shared__ int red_i[4];
  const int b = blockIdx.x;
  float s = -INFINITY;
  int i = kIdxNone;
  for (int gi = threadIdx.x; gi < a.G; gi += kThreads) {
    const float so = a.part_s[(size_t)b * a.G + gi];
    const int io = a.part_i[(size_t)b * a.G + gi];
    if (ranks_before(so, io, s, i)) { s = so; i = io; }
  }
  block_argmax(s, i, red_s, red_i);
  if (threadIdx.x == 0) {
    a.idx[b] = i == kIdxNone ? -1 : i;
    a.score[b] = s;
    write_hit(a, b, s, i);
  }
}

// k = 1 after the query-stationary kernel: the partial results name the first row of the
// 32-row block that holds a group's maximum.  Best group first (lowest block on ties), then
// the 32 rows of that one block are scored again (eight threads per row, fp32) and the best of
// them (lowest row on ties) is the answer; the score reported is the matrix-core one of phase 1.
__global__ __launch_bounds__(kThreads) void finalize_top1_block_kernel(const SearchArgs a) {
  __shared__ float red_s[4];
  __shared__ int red_i[4];
  const int b = blockIdx.x, tid = threadIdx.x;
  float s = -INFINITY;
  int i = kIdxNone;
  for (int gi = tid; gi < a.G; gi += kThreads) {
    const float so = a.part_s[(size_t)b * a.G + gi];
    const int io = a.part_i[(size_t)b * a.G + gi];
    if (ranks_before(so, io, s, i)) { s = so; i = io; }
  }
  block_argmax(s, i, red_s, red_i);
  const f16_t* q = reinterpret_cast<const f16_t*>(a.q) + (size_t)b * a.E;
  const int row = i + (tid >> 3), part = tid & 7;
  float rs = -INFINITY;
  int ri = kIdxNone;
  if (i != kIdxNone && row < a.N) {
    const f16_t* e = reinterpret_cast<const f16_t*>(a.emb) + (size_t)row * a.E;
    float acc = 0.f;
    for (int c = 8 * part; c < a.E; c += 64) {   // 16-byte pieces, eight threads side by side
      const f16x8 ev = *reinterpret_cast<const f16x8*>(e + c);
      const f16x8 qv = *reinterpret_cast<const f16x8*>(q + c);
#pragma unroll
      for (int t = 0; t < 8; ++t) acc = fmaf((float)ev[t], (float)qv[t], acc);
    }
    acc += __shfl_xor(acc, 1);
    acc += __shfl_xor(acc, 2);
    acc += __shfl_xor(acc, 4);
    rs = acc;
    ri = row;
  }
  block_argmax(rs, ri, red_s, red_i);
  if (tid == 0) {
    a.idx[b] = ri == kIdxNone ? -1 : ri;
    a.score[b] = s;
    write_hit(a, b, s, ri);
  }
}

// k > 1: pick the k best groups, re-score their rows, pick the k best rows.
// Selecting the k best of n items takes k rounds of a workgroup-wide arg-max in general; while
// the items fit one per thread (n <= 256: the common case once the groups are small) every
// thread instead counts the items that rank before its own -- the order is total, so that count
// is the item's position -- and the first k positions are written directly: one pass, two
// barriers, no rounds.
template <typename T>
__global__ __launch_bounds__(kThreads) void finalize_topk_kernel(const SearchArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* qf = reinterpret_cast<float*>(smem);          // [E]
  int* sel = reinterpret_cast<int*>(qf + a.E);         // [k] selected groups
  __shared__ float red_s[4];
  __shared__ int red_i[4];
  typedef int i32x4 __attribute__((ext_vector_type(4)));
  __shared__ __attribute__((aligned(16))) float item_s[kThreads];
  __shared__ __attribute__((aligned(16))) int item_i[kThreads];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int rpw = a.rows_per_wg;
  const T* q = reinterpret_cast<const T*>(a.q) + (size_t)b * a.E;
  for (int e = tid; e < a.E; e += kThreads) qf[e] = load_as_float(q + e);

  // position of this thread's item (s, i) among the n <= 256 items held one per thread (threads
  // without an item pass i = kIdxNone), and the number of items there are
  auto position = [&](float s, int i, int n, int& n_items) {
    item_s[tid] = s;
    item_i[tid] = i;
    __syncthreads();
    int before = 0, count = 0;
    // four items per read, no branches: every thread has stored an item (kIdxNone beyond n), so
    // reading up to the next multiple of four is safe and the extra items do not count
    for (int j = 0; j < n; j += 4) {
      const f32x4 sj = *reinterpret_cast<const f32x4*>(item_s + j);
      const i32x4 ij = *reinterpret_cast<const i32x4*>(item_i + j);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const bool there = ij[t] != kIdxNone;
        count += there ? 1 : 0;
        before += (there && ranks_before(sj[t], ij[t], s, i)) ? 1 : 0;
      }
    }
    __syncthreads();   // the arrays are used again
    n_items = count;
    return before;
  };

  // 1. the min(k, G) groups with the best maxima, in rank order
  const int ng = min(a.k, a.G);
  if (a.G <= kThreads) {
    if (tid < ng) sel[tid] = -1;   // fewer groups with a maximum than ng: the rest stay empty
    float s = -INFINITY;
    int i = kIdxNone;
    if (tid < a.G) {
      s = a.part_s[(size_t)b * a.G + tid];
      i = a.part_i[(size_t)b * a.G + tid];
    }
    int n_items;
    const int pos = position(s, i, a.G, n_items);
    if (i != kIdxNone && pos < ng) sel[pos] = i / rpw;
  } else {
    float last_s = INFINITY;
    int last_i = -1;
    for (int r = 0; r < ng; ++r) {
      float s = -INFINITY;
      int i = kIdxNone;
      for (int gi = tid; gi < a.G; gi += kThreads) {
        const float so = a.part_s[(size_t)b * a.G + gi];
        const int io = a.part_i[(size_t)b * a.G + gi];
        // only groups ranked strictly after the previous pick
        if (ranks_before(last_s, last_i, so, io) && ranks_before(so, io, s, i)) { s = so; i = io; }
      }
      block_argmax(s, i, red_s, red_i);
      if (tid == 0) sel[r] = (i == kIdxNone) ? -1 : i / rpw;
      last_s = s; last_i = i;
    }
  }
  __syncthreads();

  // 2. re-score every row of the selected groups, one row per thread -- or, when there are
  // at most 128 (64) rows, two (four) threads per row, each walking its own contiguous part: a
  // thread's walk is a chain of cache round trips, so the shorter the walk the better
  float* cand = a.cand + (size_t)b * a.k * rpw;
  const int n_rows = ng * rpw;
  const int tpr = (n_rows <= 64 && a.E % 4 == 0) ? 4 : ((n_rows <= 128 && a.E % 2 == 0) ? 2 : 1);
  if (tpr > 1) {   // one trip: thread tid takes part tid % tpr of row tid / tpr
    const int slot = tid / tpr, part = tid % tpr, seg = a.E / tpr;
    float s = 0.f;
    bool live = false;
    if (slot < n_rows) {
      const int gsel = sel[slot / rpw];
      const int r = gsel * rpw + slot % rpw;
      if (gsel >= 0 && r < a.N) {
        live = true;
        s = row_score(reinterpret_cast<const T*>(a.emb) + (size_t)r * a.E + part * seg, qf + part * seg,
                      seg, a.metric);
      }
    }
    s += __shfl_xor(s, 1);
    if (tpr == 4) s += __shfl_xor(s, 2);
    if (part == 0 && slot < n_rows) cand[slot] = live ? s : -INFINITY;
  } else
  for (int slot = tid; slot < ng * rpw; slot += kThreads) {
    const int gsel = sel[slot / rpw];
    const int r = gsel * rpw + slot % rpw;
    float s = -INFINITY;
    if (gsel >= 0 && r < a.N)
      s = row_score(reinterpret_cast<const T*>(a.emb) + (size_t)r * a.E, qf, a.E, a.metric);
    cand[slot] = s;
  }
  __syncthreads();

  // 3. the k best rows among the candidates, in rank order
  if (ng * rpw <= kThreads) {
    float s = -INFINITY;
    int i = kIdxNone;
    if (tid < ng * rpw) {
      const int gsel = sel[tid / rpw];
      const int row = gsel * rpw + tid % rpw;
      const float so = cand[tid];
      if (gsel >= 0 && row < a.N && so == so) { s = so; i = row; }   // a NaN score never ranks
    }
    int n_items;
    const int pos = position(s, i, ng * rpw, n_items);
    if (i != kIdxNone && pos < a.k) {
      a.idx[(size_t)b * a.k + pos] = i;
      a.score[(size_t)b * a.k + pos] = s;
      if (pos == 0) write_hit(a, b, s, i);
    }
    if (tid >= n_items && tid < a.k) {   // fewer rows than k ranked at all
      a.idx[(size_t)b * a.k + tid] = -1;
      a.score[(size_t)b * a.k + tid] = -INFINITY;
      if (tid == 0) write_hit(a, b, -INFINITY, kIdxNone);
    }
    return;
  }
  float last_s = INFINITY;
  int last_i = -1;
  for (int r = 0; r < a.k; ++r) {
    float s = -INFINITY;
    int i = kIdxNone;
    for (int slot = tid; slot < ng * rpw; slot += kThreads) {
      const int gsel = sel[slot / rpw];
      const int row = gsel * rpw + slot % rpw;
      if (gsel < 0 || row >= a.N) continue;
      const float so = cand[slot];
      if (ranks_before(last_s, last_i, so, row) && ranks_before(so, row, s, i)) { s = so; i = row; }
    }
    block_argmax(s, i, red_s, red_i);
    if (tid == 0) {
      a.idx[(size_t)b * a.k + r] = i == kIdxNone ? -1 : i;
      a.score[(size_t)b * a.k + r] = s;
      if (r == 0) write_hit(a, b, s, i);
    }
    last_s = s; last_i = i;
  }
}

// ------------------------------------------------------------------- host side
enum { kModeValu = 0, kModeMfma = 1, kModeMfmaBig = 2 };
constexpr int kBigBatch = 64;   // above this many queries the query-stationary kernel is used
constexpr int kBigRowsMin = 50000;   // and from this many database rows on, whatever the batch

static void search_plan(int32_t N, int32_t mode, int32_t k, int32_t* rows_per_wg, int32_t* G,
                        int32_t* wg_rows = nullptr) {
  int rpw;
  int scan = 0;   // rows per phase-1 workgroup when that is not the group
  if (mode == kModeMfma && k > 1 && N <= 32 * 1024) {
    // top-k: the second phase re-scores k whole groups per query on the vector ALUs, so the
    // groups are as small as the first phase can make them: the 32 rows of one wave.  Beyond
    // about a thousand groups the k selection rounds over the group maxima cost more than the
    // smaller groups save (140,000 rows, k = 4: 36 against 28 us).
    rpw = 32;
    scan = 128;
  } else if (mode == kModeMfma) {
    // 128 rows per pass of a workgroup; more passes per workgroup for large databases so that
    // the query tile staged in LDS is amortised, while keeping >= ~1000 workgroups
    long c = ((long)N + 128L * 1024 - 1) / (128L * 1024);
    if (c < 1) c = 1;
    if (c > 8) c = 8;
    rpw = 128 * (int)c;
  } else if (mode == kModeMfmaBig) {
    // chunks of 64 rows.  Loading the queries into registers and filling the copy pipeline
    // costs a workgroup as much as five chunks (measured), so a workgroup takes as many chunks
    // as leave about 480 workgroups: just under two per compute unit, all resident at once.  With k > 1
    // the second phase re-scores k whole groups per query, which caps the group size.
    long c = ((long)N + 64L * 480 - 1) / (64L * 480);
    if (c < 1) c = 1;
    if (c > (k > 1 ? 16 : 64)) c = k > 1 ? 16 : 64;
    rpw = kBigRows * (int)c;
  } else {
    rpw = kValuRowsPerWg;
  }
  *rows_per_wg = rpw;
  *G = (N + rpw - 1) / rpw;
  if (wg_rows) *wg_rows = scan ? scan : rpw;
}

static bool use_mfma(int32_t is_f16, int32_t metric, int32_t E) {
  return is_f16 && metric == 0 && E % 16 == 0 && E <= 512;
}

static int search_mode(int32_t is_f16, int32_t metric, int32_t E, int32_t B, int32_t N) {
  if (!use_mfma(is_f16, metric, E)) return kModeValu;
  const bool big_shape = E == 128 || E == 256 || E == 512;   // instantiated widths
  // the query-stationary kernel streams a large database faster at any batch size (1M x 256:
  // 94 us against 105-126 us for 4..64 queries); below kBigRowsMin rows both are latency-bound
  // and the row-stationary kernel starts up faster
  return (big_shape && (B > kBigBatch || N >= kBigRowsMin)) ? kModeMfmaBig : kModeMfma;
}

size_t search_workspace_bytes(int32_t N, int32_t E, int32_t B, int32_t k, int32_t is_f16) {
  // the metric is not known here: size for the larger of the paths this (dtype, E, B) can take
  size_t need = 0;
  for (int metric = 0; metric < 2; ++metric) {
    int32_t rpw, G;
    search_plan(N, search_mode(is_f16, metric, E, B, N), k, &rpw, &G);
    size_t bytes = ((size_t)B * G * 8 + 255) / 256 * 256;
    if (k > 1) bytes += (size_t)B * k * rpw * 4;
    if (bytes > need) need = bytes;
  }
  return need + 256;
}

template <int KSMAX, int QPW>
static hipError_t launch_f16_big(const SearchArgs& a, dim3 grid, hipStream_t stream) {
  hipLaunchKernelGGL((search_f16_big_kernel<KSMAX, QPW>), grid, dim3(kThreads), 0, stream, a);
  return hipGetLastError();
}

template <int KSMAX, int NQB>
static hipError_t launch_f16_one(const SearchArgs& a, dim3 grid, size_t lds, hipStream_t stream) {
  hipError_t e = ensure_lds<&search_f16_kernel<KSMAX, NQB>>(lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((search_f16_kernel<KSMAX, NQB>), grid, dim3(kThreads), lds, stream, a);
  return hipGetLastError();
}

template <int KSMAX>
static hipError_t launch_f16_phase1(const SearchArgs& a, int nqb, dim3 grid, size_t lds,
                                    hipStream_t stream) {
  switch (nqb) {
    case 1: return launch_f16_one<KSMAX, 1>(a, grid, lds, stream);
    case 2: return launch_f16_one<KSMAX, 2>(a, grid, lds, stream);
    case 4: return launch_f16_one<KSMAX, 4>(a, grid, lds, stream);
    default: return launch_f16_one<KSMAX, 8>(a, grid, lds, stream);
  }
}

static size_t f16_lds_bytes(int nqb, int E) {
  return (size_t)32 * nqb * (E + kQPad) * 2 + (size_t)4 * 32 * nqb * 8;
}

hipError_t launch_search(const SearchLaunch& p, hipStream_t stream) {
  if (p.B == 0) return hipSuccess;
  SearchArgs a;
  a.emb = p.emb; a.q = p.q; a.map_of = p.map_of;
  a.N = p.N; a.E = p.E; a.B = p.B; a.k = p.k; a.metric = p.metric;
  a.threshold = p.threshold;
  a.idx = p.idx; a.score = p.score; a.hit = p.hit;
  const int mode = search_mode(p.is_f16, p.metric, p.E, p.B, p.N);
  const bool mfma = mode == kModeMfma;
  search_plan(p.N, mode, p.k, &a.rows_per_wg, &a.G, &a.wg_rows);
  unsigned char* ws = reinterpret_cast<unsigned char*>(p.ws);
  size_t part_bytes = ((size_t)p.B * a.G * 8 + 255) / 256 * 256;
  a.part_s = reinterpret_cast<float*>(ws);
  a.part_i = reinterpret_cast<int32_t*>(ws + (size_t)p.B * a.G * 4);
  a.cand = reinterpret_cast<float*>(ws + part_bytes);
  a.q0 = 0; a.nq = p.B;

  if (mode == kModeMfmaBig) {
    // query super-blocks of 128 * QPW queries (4 waves x QPW blocks of 32); two blocks per wave
    // only while the query operands fit in the register file (E <= 256)
    const int ksmax = p.E <= 128 ? 8 : (p.E <= 256 ? 16 : 32);
    const int qpw_max = p.E <= 256 ? 2 : 1;
    const dim3 grid((unsigned)a.G);
    for (int q0 = 0; q0 < p.B; q0 += 128 * qpw_max) {
      a.q0 = q0;
      a.nq = p.B - q0 < 128 * qpw_max ? p.B - q0 : 128 * qpw_max;
      const int qpw = a.nq > 128 ? 2 : 1;
      hipError_t e;
      if (ksmax == 8) e = qpw == 2 ? launch_f16_big<8, 2>(a, grid, stream) : launch_f16_big<8, 1>(a, grid, stream);
      else if (ksmax == 16) e = qpw == 2 ? launch_f16_big<16, 2>(a, grid, stream) : launch_f16_big<16, 1>(a, grid, stream);
      else e = launch_f16_big<32, 1>(a, grid, stream);
      if (e != hipSuccess) return e;
    }
  } else if (mfma) {
    // query super-blocks of 32 * nqb queries; the staged tile must fit in LDS
    const int ksmax = p.E <= 128 ? 8 : (p.E <= 256 ? 16 : 32);
    int max_nqb = 8;
    while (max_nqb > 1 && f16_lds_bytes(max_nqb, p.E) > 150 * 1024) max_nqb >>= 1;
    for (int q0 = 0; q0 < p.B; q0 += 32 * max_nqb) {
      a.q0 = q0;
      a.nq = p.B - q0 < 32 * max_nqb ? p.B - q0 : 32 * max_nqb;
      int nqb = 1;
      while (32 * nqb < a.nq) nqb <<= 1;
      const size_t lds = f16_lds_bytes(nqb, p.E);
      const dim3 grid((unsigned)((p.N + a.wg_rows - 1) / a.wg_rows));
      hipError_t e;
      if (ksmax == 8) e = launch_f16_phase1<8>(a, nqb, grid, lds, stream);
      else if (ksmax == 16) e = launch_f16_phase1<16>(a, nqb, grid, lds, stream);
      else e = launch_f16_phase1<32>(a, nqb, grid, lds, stream);
      if (e != hipSuccess) return e;
    }
  } else {
    const dim3 grid((unsigned)a.G, (unsigned)p.B);
    const size_t lds = (size_t)p.E * 4;
    if (p.is_f16) hipLaunchKernelGGL((search_valu_kernel<f16_t>), grid, dim3(kThreads), lds, stream, a);
    else hipLaunchKernelGGL((search_valu_kernel<float>), grid, dim3(kThreads), lds, stream, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }

  if (p.k == 1 && mode == kModeMfmaBig) {
    hipLaunchKernelGGL(finalize_top1_block_kernel, dim3((unsigned)p.B), dim3(kThreads), 0, stream, a);
  } else if (p.k == 1) {
    hipLaunchKernelGGL(finalize_top1_kernel, dim3((unsigned)p.B), dim3(kThreads), 0, stream, a);
  } else {
    const size_t lds = (size_t)p.E * 4 + (size_t)p.k * 4;
    if (p.is_f16) hipLaunchKernelGGL((finalize_topk_kernel<f16_t>), dim3((unsigned)p.B), dim3(kThreads), lds, stream, a);
    else hipLaunchKernelGGL((finalize_topk_kernel<float>), dim3((unsigned)p.B), dim3(kThreads), lds, stream, a);
  }
  return hipGetLastError();
}

}  // namespace ac
