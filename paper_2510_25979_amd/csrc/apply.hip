// Reuse branch of Algorithm 2: O = A_cached . V, with the cached map read in
// place from the database (the hit index selects the entry; nothing is
// gathered or copied first).
//
// bf16 path (matrix cores).  One workgroup = one (query, layer, head group,
// block of 128 map rows); a wave owns 32 map rows.  The product is formed
// transposed, O^T = V^T A^T, so that
//   - the map operand (columns of A^T = rows of A) is eight consecutive bf16
//     of one map row per lane: a plain 16-byte global load, no LDS;
//   - the V operand comes from an LDS tile that was transposed while staging;
//   - each lane ends up with runs of four consecutive d of one output row.
// Causal maps are exactly zero above the diagonal, so a wave reads only the
// column range [0, last row of its block]; nothing above is fetched.
// HBM-bound: per (query, layer, head) the kernel moves about S(S+32) map
// bytes... (bf16: 2 bytes each) plus V and O once.
#include "common.hpp"
#include "launch.hpp"

namespace ac {

struct ApplyArgs {
  const void* maps;     // [M][L][Hq][S][S] (device), or one staged entry
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

template <int D, bool CAUSAL>
__global__ __launch_bounds__(kThreads, 2) void apply_bf16_kernel(const ApplyArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* vt = reinterpret_cast<bf16_t*>(smem);                 // [D][kVtStride]
  bf16_t* ost_all = vt + D * kVtStride;                          // [4][32][D + 4]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int il = lane & 31, kh = lane >> 5;

  // Block id -> (tile, row block).  The eight row blocks... of one tile share V, and
  // workgroups are handed to the 8 XCDs round-robin by id, so ids that differ
  // by a multiple of 8 (same XCD, same L2) are given to one tile.
  const int bid = blockIdx.x;
  const int tile = (bid >> 3) / a.n_rblk * 8 + (bid & 7);
  const int rblk = a.n_rblk - 1 - (bid >> 3) % a.n_rblk;   // heaviest row block first
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
  const bf16_t* Vt_src = reinterpret_cast<const bf16_t*>(a.V) +
                         (((size_t)b * a.Lc + l) * a.Hkv + kvh) * (size_t)S * D;
  const size_t layer_stride = (size_t)a.Hq * S * S;
  const bf16_t* A_layer = reinterpret_cast<const bf16_t*>(a.maps) +
                          ((size_t)entry * a.L + (a.layer_begin + l)) * layer_stride;

  const int r0 = rblk * kChunk + wave * kRowsPerWave;   // first map row of this wave
  const bool active = r0 < S;
  const int n_chunk = CAUSAL ? rblk + 1 : (S + kChunk - 1) / kChunk;

  for (int hl = 0; hl < a.heads_per_wg; ++hl) {
    const int h = h0 + hl;
    const bf16_t* Arow = A_layer + (size_t)h * S * S + (size_t)(r0 + il) * S + 8 * kh;
    f32x16 acc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;

    for (int c = 0; c < n_chunk; ++c) {
      const int j0 = c * kChunk;
      const int nj = min(kChunk, S - j0);
      // columns this wave needs from the chunk (multiple of 32; causal: up to its last row)
      int ncol = active ? nj : 0;
      if (CAUSAL && active) ncol = min(nj, r0 + kRowsPerWave - j0);
      const int nks = ncol >> 4;

      // 1. issue the map loads first: they stay in flight while V is staged
      bf16x8 am[8];
#pragma unroll
      for (int ks = 0; ks < 8; ++ks)
        if (ks < nks) am[ks] = *reinterpret_cast<const bf16x8*>(Arow + j0 + 16 * ks);

      // 2. stage V^T for this chunk (once per workgroup; shared by its heads)
      if (hl == 0 || n_chunk > 1) {
        if (c > 0 || hl > 0) __syncthreads();
        stage_v_transposed<D>(Vt_src + (size_t)j0 * D, nj, vt, tid);
        __syncthreads();
      }

      // 3. O^T[d][i] += sum_j V^T[d][j] A^T[j][i]
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        if (ks < nks) {
#pragma unroll
          for (int db = 0; db < D / 32; ++db) {
            const u32x2* src =
                reinterpret_cast<const u32x2*>(vt + (32 * db + il) * kVtStride + 16 * ks + 8 * kh);
            u32x2 lo = src[0], hi = src[1];
            u32x4 w = {lo.x, lo.y, hi.x, hi.y};
            acc[db] = mfma_bf16(__builtin_bit_cast(bf16x8, w), am[ks], acc[db]);
          }
        }
      }
    }

    if (active) {
      bf16_t* dst = reinterpret_cast<bf16_t*>(a.O) +
                    ((((size_t)b * a.Lc + l) * a.Hq + h) * S + r0) * (size_t)D;
      store_tile_bf16<D>(acc, 1.0f, ost_all + wave * (32 * (D + 4)), dst, lane);
    }
  }
}

// fp32 path (vector ALUs): small, correctness-first kernel for fp32 databases.
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
  const size_t lds = apply_lds_bytes(p.D);
#define AC_LAUNCH_APPLY(DD, CC)                                                              \
  do {                                                                                       \
    hipError_t e = ensure_lds<&apply_bf16_kernel<DD, CC>>(lds);                              \
    if (e != hipSuccess) return e;                                                           \
    hipLaunchKernelGGL((apply_bf16_kernel<DD, CC>), grid, dim3(kThreads), lds, stream, a);   \
  } while (0)
  if (p.D == 64) {
    if (p.causal) AC_LAUNCH_APPLY(64, true); else AC_LAUNCH_APPLY(64, false);
  } else {
    if (p.causal) AC_LAUNCH_APPLY(128, true); else AC_LAUNCH_APPLY(128, false);
  }
#undef AC_LAUNCH_APPLY
  return hipGetLastError();
}

}  // namespace ac
