// Recompute branch of Algorithm 2: O = softmax(scale * Q K^T) V, causal or
// dense, without ever writing the S x S map (flash-style online softmax).
//
// bf16 path (matrix cores).  One workgroup = one (batch item, query head,
// block of 128 query rows); a wave owns 32 query rows and walks the key
// blocks up to its diagonal.  Both products are formed transposed:
//   S^T = K Q^T   -> a lane holds 16 keys of ONE query column, so the row
//                    maximum and row sum are in-lane reductions plus one
//                    exchange between the two lane halves;
//   O^T = V^T P^T -> the probabilities sit in exactly the register layout
//                    the second product wants as its column operand, so P
//                    goes from the first MFMA to the second without leaving
//                    registers (the contraction slots are matched by reading
//                    V^T from LDS in the same key order).
// K is staged row-major, V transposed, 128 keys per LDS chunk.
#include "common.hpp"
#include "launch.hpp"

namespace ac {

constexpr int kKPad = 8;   // elements of padding per staged K row (keeps 16-byte alignment)

struct ExactArgs {
  const void *Q, *K, *V;
  void* O;
  const int32_t* row_sel;
  int32_t B, Hq, Hkv, S;
  int32_t n_rblk;     // ceil(S / 128)
  int32_t n_kvtiles;  // B * Hkv
  float scale_log2e;  // scale * log2(e): softmax is evaluated with exp2
};

template <int D, bool CAUSAL>
__global__ __launch_bounds__(kThreads, 2) void exact_bf16_kernel(const ExactArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int KS = D + kKPad;                       // staged K row stride (elements)
  bf16_t* ks_lds = reinterpret_cast<bf16_t*>(smem);  // [128][KS]; reused for the output tile
  bf16_t* vt = ks_lds + kChunk * KS;                  // [D][kVtStride]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int il = lane & 31, kh = lane >> 5;
  const int S = a.S, g = a.Hq / a.Hkv;

  // Block id -> (kv tile u, head within its group, row block).  All blocks that
  // share K and V (the g heads of a group and their row blocks) get ids that
  // are equal mod 8, i.e. the same XCD and L2.
  const int bid = blockIdx.x;
  const int slot = bid >> 3;
  const int per_u = g * a.n_rblk;
  const int u = (slot / per_u) * 8 + (bid & 7);
  if (u >= a.n_kvtiles) return;
  const int hl = (slot % per_u) / a.n_rblk;
  const int rblk = a.n_rblk - 1 - (slot % per_u) % a.n_rblk;   // heaviest row block first
  const int b = u / a.Hkv, kvh = u % a.Hkv;
  const int h = kvh * g + hl;
  if (a.row_sel && a.row_sel[b] >= 0) return;   // served by the reuse branch

  const bf16_t* Qt = reinterpret_cast<const bf16_t*>(a.Q) + ((size_t)b * a.Hq + h) * (size_t)S * D;
  const bf16_t* Kt = reinterpret_cast<const bf16_t*>(a.K) + (size_t)u * S * D;
  const bf16_t* Vt_src = reinterpret_cast<const bf16_t*>(a.V) + (size_t)u * S * D;

  const int r0 = rblk * kChunk + wave * kRowsPerWave;
  const bool active = r0 < S;

  // query operand: lane (il, kh) keeps Q[r0 + il][16 ks + 8 kh .. +8) for every ks
  bf16x8 qreg[D / 16];
  if (active) {
    const bf16_t* qrow = Qt + (size_t)(r0 + il) * D + 8 * kh;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) qreg[ks] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ks);
  } else {
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks)
#pragma unroll
      for (int e = 0; e < 8; ++e) qreg[ks][e] = (bf16_t)0.f;
  }

  f32x16 acc[D / 32];
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[db][v] = 0.f;
  float m_run = -INFINITY;   // running maximum of scaled logits (log2 domain), per query column
  float l_run = 0.f;         // this lane's share of the running sum

  const int n_chunk = CAUSAL ? rblk + 1 : (S + kChunk - 1) / kChunk;
  for (int c = 0; c < n_chunk; ++c) {
    const int j0 = c * kChunk;
    const int nj = min(kChunk, S - j0);
    if (c > 0) __syncthreads();
    // stage K rows (16-byte pieces, row-major) and V transposed
    {
      constexpr int DQ = D / 8;
      const u32x4* src = reinterpret_cast<const u32x4*>(Kt + (size_t)j0 * D);
      for (int p = tid; p < nj * DQ; p += kThreads) {
        const int j = p / DQ, dq = p % DQ;
        *reinterpret_cast<u32x4*>(ks_lds + j * KS + 8 * dq) = src[p];
      }
    }
    stage_v_transposed<D>(Vt_src + (size_t)j0 * D, nj, vt, tid);
    __syncthreads();

    if (active) {
      int nblk = nj >> 5;                                   // 32-key blocks in this chunk
      if (CAUSAL) nblk = min(nblk, (r0 - j0) / 32 + 1);     // up to the diagonal block
      for (int jb = 0; jb < nblk; ++jb) {
        // S^T block: 32 keys x 32 queries
        f32x16 s;
#pragma unroll
        for (int v = 0; v < 16; ++v) s[v] = 0.f;
        const bf16_t* krow = ks_lds + (32 * jb + il) * KS + 8 * kh;
#pragma unroll
        for (int ks = 0; ks < D / 16; ++ks) {
          bf16x8 kop = *reinterpret_cast<const bf16x8*>(krow + 16 * ks);
          s = mfma_bf16(kop, qreg[ks], s);
        }
        // scaled logits in the log2 domain, mask above the diagonal
        const bool diag = CAUSAL && (j0 + 32 * jb == r0);
        float mx = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float t = s[v] * a.scale_log2e;
          if (diag && mfma_row(v, kh) > il) t = -INFINITY;
          s[v] = t;
          mx = fmaxf(mx, t);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);   // finite: key 0 is visible to every query
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        m_run = m_new;
        float psum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          s[v] = __builtin_amdgcn_exp2f(s[v] - m_new);
          psum += s[v];
        }
        l_run = l_run * alpha + psum;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[db][v] *= alpha;
        // O^T += V^T P^T; contraction slot (kh, e) of step s2 is key
        // 32 jb + 16 s2 + 8 (e / 4) + 4 kh + e % 4, the key of result register 8 s2 + e
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          u32x4 pw;
          pw.x = pack_bf16(s[8 * s2 + 0], s[8 * s2 + 1]);
          pw.y = pack_bf16(s[8 * s2 + 2], s[8 * s2 + 3]);
          pw.z = pack_bf16(s[8 * s2 + 4], s[8 * s2 + 5]);
          pw.w = pack_bf16(s[8 * s2 + 6], s[8 * s2 + 7]);
          const bf16x8 pop = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
          for (int db = 0; db < D / 32; ++db) {
            const bf16_t* vrow = vt + (32 * db + il) * kVtStride + 32 * jb + 16 * s2 + 4 * kh;
            u32x2 lo = *reinterpret_cast<const u32x2*>(vrow);
            u32x2 hi = *reinterpret_cast<const u32x2*>(vrow + 8);
            u32x4 w = {lo.x, lo.y, hi.x, hi.y};
            acc[db] = mfma_bf16(__builtin_bit_cast(bf16x8, w), pop, acc[db]);
          }
        }
      }
    }
  }

  __syncthreads();   // every wave is done with the staged K: reuse it for the output tile
  if (active) {
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    bf16_t* dst = reinterpret_cast<bf16_t*>(a.O) + (((size_t)b * a.Hq + h) * S + r0) * (size_t)D;
    store_tile_bf16<D>(acc, 1.0f / l_tot, ks_lds + wave * (32 * (D + 4)), dst, lane);
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
  const int nj = causal ? i + 1 : S;
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

static size_t exact_lds_bytes(int D) {
  return (size_t)(kChunk * (D + kKPad) + D * kVtStride) * sizeof(bf16_t);
}

hipError_t launch_exact(const ExactLaunch& p, hipStream_t stream) {
  if (p.B == 0) return hipSuccess;
  ExactArgs a;
  a.Q = p.Q; a.K = p.K; a.V = p.V; a.O = p.O; a.row_sel = p.row_sel;
  a.B = p.B; a.Hq = p.Hq; a.Hkv = p.Hkv; a.S = p.S;
  a.n_rblk = (p.S + kChunk - 1) / kChunk;
  a.n_kvtiles = p.B * p.Hkv;
  const float scale = p.scale == 0.f ? 1.0f / sqrtf((float)p.D) : p.scale;
  a.scale_log2e = scale * 1.44269504088896340736f;
  if (p.is_f32) {
    const unsigned blocks = (unsigned)((size_t)p.B * p.Hq * p.S);
    hipLaunchKernelGGL(exact_f32_kernel, dim3(blocks), dim3(kWave), (size_t)p.S * sizeof(float),
                       stream, a, p.D, p.causal, scale);
    return hipGetLastError();
  }
  const int g = p.Hq / p.Hkv;
  const int u8 = (a.n_kvtiles + 7) / 8 * 8;
  const dim3 grid((unsigned)((size_t)u8 * g * a.n_rblk));
  const size_t lds = exact_lds_bytes(p.D);
#define AC_LAUNCH_EXACT(DD, CC)                                                              \
  do {                                                                                       \
    hipError_t e = ensure_lds<&exact_bf16_kernel<DD, CC>>(lds);                              \
    if (e != hipSuccess) return e;                                                           \
    hipLaunchKernelGGL((exact_bf16_kernel<DD, CC>), grid, dim3(kThreads), lds, stream, a);   \
  } while (0)
  if (p.D == 64) {
    if (p.causal) AC_LAUNCH_EXACT(64, true); else AC_LAUNCH_EXACT(64, false);
  } else {
    if (p.causal) AC_LAUNCH_EXACT(128, true); else AC_LAUNCH_EXACT(128, false);
  }
#undef AC_LAUNCH_EXACT
  return hipGetLastError();
}

}  // namespace ac
