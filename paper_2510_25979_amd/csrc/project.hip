// Feature projector (AttnCache Algorithm 1, f = feature_projector(h); Sec. 3.1
// "Feature Projector": two MLP layers that lower the dimension of the input
// embedding).  Four small kernels, all in binary32:
//
//   pool_kernel     x[b][i]  = mean over the sentence's tokens of h[b][t][i]      HBM-bound
//   dense_kernel    P1[z]    = partial products of x with W1 over K-slice z       fp32 matrix cores
//   dense_kernel    P2[z]    = partial products of relu(b1 + sum_z P1[z]) with W2
//   finish_kernel   f[b]     = b2 + sum_z P2[z], optionally scaled to unit norm, cast
//
// The two layers are dense contractions, so they run on the matrix cores
// (v_mfma_f32_32x32x2_f32: full binary32 operands, same peak as the vector
// ALUs but no staging through LDS: operands go from global memory straight
// into the lanes that feed the instruction).  With 64 queries a layer has only
// a few dozen 32 x 32 output tiles, so the contraction index is split over
// workgroups and the slices are added, in slice order, by whoever reads them
// next: the result does not depend on scheduling.  Most of the split happens
// inside a workgroup (up to 16 waves, partial tiles added through LDS), so few
// partial results travel through global memory.
#include <algorithm>
#include <type_traits>

#include "common.hpp"
#include "launch.hpp"

namespace ac {
namespace {

constexpr int kPoolWaves = 8;

// Intermediate activations (pooled input, partial layer outputs) are stored as
// [index / 4][query][4]: the 16-byte piece a lane of the dense kernel wants
// (four consecutive contraction indices of its query) sits next to the pieces
// of the neighbouring queries, so one load instruction of a wave touches 8
// cache lines instead of 32 (a row-major [query][index] array made the dense
// kernel's load phase 2.5 times longer).
__device__ __forceinline__ size_t granule_at(int index4, int b, int B) {
  return ((size_t)index4 * B + b) * 4;
}

// ---- pooling ---------------------------------------------------------------
// grid (ceil(dm / (64 * VEC)), B), kPoolWaves waves.  Wave w adds tokens w,
// w + kPoolWaves, ...; a lane owns VEC consecutive columns (one 16-byte load
// per token).  The waves' partial sums meet in LDS and are added in wave order.
template <typename T> struct PoolVec;
template <> struct PoolVec<bf16_t> { static constexpr int VEC = 8; };
template <> struct PoolVec<float> { static constexpr int VEC = 4; };

template <int VEC>
__device__ __forceinline__ void pool_add(float (&acc)[VEC], u32x4 w);
template <>
__device__ __forceinline__ void pool_add<8>(float (&acc)[8], u32x4 w) {
#pragma unroll
  for (int p = 0; p < 4; ++p) {   // a bf16 is the upper half of the binary32 of the same value
    acc[2 * p] += __builtin_bit_cast(float, w[p] << 16);
    acc[2 * p + 1] += __builtin_bit_cast(float, w[p] & 0xffff0000u);
  }
}
template <>
__device__ __forceinline__ void pool_add<4>(float (&acc)[4], u32x4 w) {
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const uint32_t bits = w[p];   // a copy: the cast wants an object, not a vector element
    acc[p] += __builtin_bit_cast(float, bits);
  }
}

template <typename T>
__global__ __launch_bounds__(kPoolWaves * kWave) void pool_kernel(const T* __restrict__ h,
                                                        const int32_t* __restrict__ seq_len,
                                                        float* __restrict__ x, int S, int dm,
                                                        int B) {
  constexpr int VEC = PoolVec<T>::VEC;
  constexpr int UNROLL = 16;
  __shared__ float part[kPoolWaves][kWave * VEC];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = blockIdx.y;
  const int col = (blockIdx.x * kWave + lane) * VEC;
  int s = seq_len ? seq_len[b] : S;
  s = min(max(s, 1), S);
  float acc[VEC];
#pragma unroll
  for (int v = 0; v < VEC; ++v) acc[v] = 0.f;
  if (col < dm) {
    const T* src = h + (size_t)b * S * dm + col;
    // every load of a round is issued before the first sum: one memory round trip per round
    for (int t = wave; t < s; t += kPoolWaves * UNROLL) {
      u32x4 w[UNROLL];
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        const int tt = t + kPoolWaves * u;   // wave-uniform, so the test costs no lanes
        w[u] = u32x4{0u, 0u, 0u, 0u};
        if (tt < s)
          w[u] = __builtin_nontemporal_load(
              reinterpret_cast<const u32x4*>(src + (size_t)tt * dm));
      }
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) pool_add<VEC>(acc, w[u]);
    }
  }
#pragma unroll
  for (int v = 0; v < VEC; ++v) part[wave][lane * VEC + v] = acc[v];
  __syncthreads();
  if (wave == 0 && col < dm) {
    const float fs = (float)s;
    float out[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
      float sum = part[0][lane * VEC + v];
#pragma unroll
      for (int w = 1; w < kPoolWaves; ++w) sum += part[w][lane * VEC + v];
      out[v] = sum / fs;
    }
#pragma unroll
    for (int v = 0; v < VEC; v += 4) {
      f32x4 o = {out[v], out[v + 1], out[v + 2], out[v + 3]};
      *reinterpret_cast<f32x4*>(x + granule_at((col + v) >> 2, b, B)) = o;
    }
  }
}

// ---- one dense layer, split over the contraction index ----------------------
// out[z][b][j] = sum over k in slice z of  W[j][k] * in(b, k),
// in(b, k) = act(bias_in[k] + sum_{zi < NZ_IN} in_part[zi][b][k]),
// act = max(0, .) when RELU (the input and activation of a layer are compile-time
// cases so that no branch sits between the loads).
// grid (ceil(J / 32), ceil(B / 32), nz), up to 16 waves per workgroup.  The
// workgroup owns a 32 (j) x 32 (b) tile and K-slice z; its waves split that
// slice further, each forms its own 32 x 32 partial tile on the matrix core,
// and the partial tiles are added through LDS in wave order.
// v_mfma_f32_32x32x2_f32 takes from lane l one element of row l % 32 at
// contraction slot l / 32; a lane loads four consecutive k of its row in one
// 16-byte load (k = k0 + 4 (l / 32) + t feeds product t), which is a valid
// assignment of indices to slots because W and the input use the same one.
// K, the per-wave slice length and J are multiples of 8.
constexpr int kDenseWaves = 16;

struct DenseArgs {
  const float* W;        // [J][K]
  const float* in_part;  // [NZ_IN][K / 4][B][4]
  const float* bias_in;  // [K] or nullptr
  float* out;            // [nz][J / 4][B][4]
  int B, J, K, slice;    // slice: contraction indices per wave
};

// Loads of one step of a lane (eight contraction indices of the tile, four of
// them this lane's): its piece of W, of each of the NZ_IN partial inputs and
// of the bias.  Requested together; combined only after a scheduling fence so
// that a step costs one memory round trip, not one per operand.
template <int NZ_IN>
struct DenseRaw {
  f32x4 w, part[NZ_IN], bias;
};

template <int NZ_IN, bool BIAS>
__device__ __forceinline__ DenseRaw<NZ_IN> dense_load(const DenseArgs& a, const float* wrow, int b,
                                                      int k, int kh) {
  DenseRaw<NZ_IN> r;
  r.w = *reinterpret_cast<const f32x4*>(wrow + k);
  const size_t at = granule_at((k >> 2) + kh, b, a.B);
  const size_t zstride = (size_t)a.B * a.K;
#pragma unroll
  for (int z = 0; z < NZ_IN; ++z)
    r.part[z] = *reinterpret_cast<const f32x4*>(a.in_part + z * zstride + at);
  if (BIAS) r.bias = *reinterpret_cast<const f32x4*>(a.bias_in + k + 4 * kh);
  return r;
}

template <int NZ_IN, bool BIAS, bool RELU>
__device__ __forceinline__ f32x4 dense_input(const DenseRaw<NZ_IN>& r) {
  f32x4 v = r.part[0];
#pragma unroll
  for (int z = 1; z < NZ_IN; ++z) v += r.part[z];
  if (BIAS) v += r.bias;
  if (RELU) {
#pragma unroll
    for (int t = 0; t < 4; ++t) v[t] = fmaxf(v[t], 0.f);
  }
  return v;
}

template <int NZ_IN, bool BIAS, bool RELU>
__global__ __launch_bounds__(kDenseWaves * kWave) void dense_kernel(DenseArgs a) {
  __shared__ float red[kDenseWaves][16][kWave];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_waves = blockDim.x >> 6;
  const int r = lane & 31, kh = lane >> 5;
  const int j0 = 32 * blockIdx.x, b0 = 32 * blockIdx.y;
  const int k_begin = min((blockIdx.z * n_waves + wave) * a.slice, a.K);
  const int k_end = min(k_begin + a.slice, a.K);
  // rows past the edge repeat the last one; their products are never stored
  const int jr = min(j0 + r, a.J - 1), br = min(b0 + r, a.B - 1);
  const float* wrow = a.W + (size_t)jr * a.K + 4 * kh;
  f32x16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.f;
  int k = k_begin;
  for (; k + 32 <= k_end; k += 32) {
    DenseRaw<NZ_IN> raw[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) raw[u] = dense_load<NZ_IN, BIAS>(a, wrow, br, k + 8 * u, kh);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const f32x4 x = dense_input<NZ_IN, BIAS, RELU>(raw[u]);
#pragma unroll
      for (int t = 0; t < 4; ++t)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(raw[u].w[t], x[t], acc, 0, 0, 0);
    }
  }
  for (; k < k_end; k += 8) {
    const DenseRaw<NZ_IN> raw = dense_load<NZ_IN, BIAS>(a, wrow, br, k, kh);
    const f32x4 x = dense_input<NZ_IN, BIAS, RELU>(raw);
#pragma unroll
    for (int t = 0; t < 4; ++t)
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(raw.w[t], x[t], acc, 0, 0, 0);
  }
  // a lane holds query b0 + r; its register v holds output j0 + mfma_row(v, kh)
#pragma unroll
  for (int v = 0; v < 16; ++v) red[wave][v][lane] = acc[v];
  __syncthreads();
  // 256 items per tile: (vq, lane) -> four consecutive outputs of one query
  for (int item = tid; item < 4 * kWave; item += blockDim.x) {
    const int vq = item >> 6, l = item & 63;
    const int b = b0 + (l & 31), j = j0 + 8 * vq + 4 * (l >> 5);
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
    for (int w = 0; w < n_waves; ++w)
#pragma unroll
      for (int t = 0; t < 4; ++t) o[t] += red[w][4 * vq + t][l];
    if (b < a.B && j < a.J)
      *reinterpret_cast<f32x4*>(a.out + (size_t)blockIdx.z * a.B * a.J + granule_at(j >> 2, b, a.B)) = o;
  }
}

// ---- bias, unit norm, cast ---------------------------------------------------
// grid B, 256 threads; thread t owns outputs t, t + 256, ...
template <typename OUT>
__global__ __launch_bounds__(kThreads) void finish_kernel(const float* __restrict__ part, int nz,
                                                          const float* __restrict__ bias,
                                                          OUT* __restrict__ feat, int B, int E,
                                                          int normalize) {
  __shared__ float wsum[kThreads / kWave];
  const int b = blockIdx.x, tid = threadIdx.x;
  constexpr int kMaxOwn = 8;   // E <= 2048
  float val[kMaxOwn];
  float sq = 0.f;
#pragma unroll
  for (int o = 0; o < kMaxOwn; ++o) {
    const int e = tid + o * kThreads;
    float v = 0.f;
    if (e < E) {
      v = bias ? bias[e] : 0.f;
      for (int z = 0; z < nz; ++z) v += part[(size_t)z * B * E + granule_at(e >> 2, b, B) + (e & 3)];
    }
    val[o] = v;
    sq += v * v;
  }
  float mul = 1.f;
  if (normalize) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sq += __shfl_xor(sq, off);
    if ((tid & 63) == 0) wsum[tid >> 6] = sq;
    __syncthreads();
    const float total = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
    if (total > 0.f) mul = 1.f / sqrtf(total);
  }
#pragma unroll
  for (int o = 0; o < kMaxOwn; ++o) {
    const int e = tid + o * kThreads;
    if (e < E) feat[(size_t)b * E + e] = (OUT)(val[o] * mul);
  }
}

int ceil_div(int a, int b) { return (a + b - 1) / b; }

// How one layer's contraction index is split: waves per workgroup, workgroups
// along K (= partial results in global memory) and indices per wave.  Aim: about
// one wave per SIMD of the chip (1024), at least 32 indices per wave.
struct DenseSplit { int n_waves, nz, slice; };
DenseSplit dense_split(int32_t B, int32_t J, int32_t K) {
  const int tiles = ceil_div(B, 32) * ceil_div(J, 32);
  // waves per tile: about two per SIMD of the chip in total, 32 indices each at least
  const int want = std::min(std::max(1, 2048 / tiles), std::min(std::max(1, K / 32), 64));
  // Spread them over workgroups first (more compute units share the load phase), up to the
  // four partial results the next kernel reads, then over the waves of a workgroup.
  DenseSplit d;
  d.nz = std::min(want, 4);
  if (d.nz == 3) d.nz = 2;
  d.n_waves = std::min(ceil_div(want, d.nz), kDenseWaves);
  d.slice = ceil_div(ceil_div(K, d.n_waves * d.nz), 8) * 8;
  return d;   // slices past K are empty and contribute zeros
}

}  // namespace

size_t project_workspace_bytes(int32_t B, int32_t dm, int32_t hid, int32_t E) {
  const DenseSplit s1 = dense_split(B, hid, dm), s2 = dense_split(B, E, hid);
  return sizeof(float) * ((size_t)B * dm + (size_t)s1.nz * B * hid + (size_t)s2.nz * B * E);
}

hipError_t launch_project(const ProjectLaunch& p, hipStream_t stream) {
  const DenseSplit s1 = dense_split(p.B, p.hid, p.dm), s2 = dense_split(p.B, p.E, p.hid);
  float* x = static_cast<float*>(p.ws);
  float* p1 = x + (size_t)p.B * p.dm;
  float* p2 = p1 + (size_t)s1.nz * p.B * p.hid;

  if (p.h_is_f32) {
    dim3 grid(ceil_div(p.dm, kWave * 4), p.B);
    pool_kernel<float><<<grid, kPoolWaves * kWave, 0, stream>>>(static_cast<const float*>(p.h),
                                                                p.seq_len, x, p.S, p.dm, p.B);
  } else {
    dim3 grid(ceil_div(p.dm, kWave * 8), p.B);
    pool_kernel<bf16_t><<<grid, kPoolWaves * kWave, 0, stream>>>(static_cast<const bf16_t*>(p.h),
                                                                 p.seq_len, x, p.S, p.dm, p.B);
  }
  DenseArgs l1{p.W1, x, nullptr, p1, p.B, p.hid, p.dm, s1.slice};
  dense_kernel<1, false, false><<<dim3(ceil_div(p.hid, 32), ceil_div(p.B, 32), s1.nz),
                                  s1.n_waves * kWave, 0, stream>>>(l1);
  DenseArgs l2{p.W2, p1, p.b1, p2, p.B, p.E, p.hid, s2.slice};
  const dim3 grid2(ceil_div(p.E, 32), ceil_div(p.B, 32), s2.nz);
  const int threads2 = s2.n_waves * kWave;
  auto layer2 = [&](auto nz_in) {
    constexpr int NZ = decltype(nz_in)::value;
    if (p.b1)
      dense_kernel<NZ, true, true><<<grid2, threads2, 0, stream>>>(l2);
    else
      dense_kernel<NZ, false, true><<<grid2, threads2, 0, stream>>>(l2);
  };
  switch (s1.nz) {
    case 1: layer2(std::integral_constant<int, 1>{}); break;
    case 2: layer2(std::integral_constant<int, 2>{}); break;
    default: layer2(std::integral_constant<int, 4>{}); break;
  }
  if (p.feat_is_f16)
    finish_kernel<f16_t><<<p.B, kThreads, 0, stream>>>(p2, s2.nz, p.b2, static_cast<f16_t*>(p.feat),
                                                       p.B, p.E, p.normalize);
  else
    finish_kernel<float><<<p.B, kThreads, 0, stream>>>(p2, s2.nz, p.b2, static_cast<float*>(p.feat),
                                                       p.B, p.E, p.normalize);
  return hipGetLastError();
}

}  // namespace ac
