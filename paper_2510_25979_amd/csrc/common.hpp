// Shared device-side helpers of the gfx950 kernels: vector types, matrix-core
// (MFMA) wrappers, bf16 conversion, LDS staging of a transposed V tile.
//
// Matrix-core data layout used throughout (wave64, v_mfma_f32_32x32x16_*):
//   operand A (32 x 16): lane l supplies row (l % 32), eight consecutive
//                        k-slots starting at 8 * (l / 32);
//   operand B (16 x 32): lane l supplies column (l % 32), same k-slots;
//   result   (32 x 32): lane l holds column (l % 32); register v (0..15)
//                        holds row 8 * (v / 4) + 4 * (l / 32) + (v % 4).
// k-slot s of A is multiplied with k-slot s of B, so any assignment of real
// contraction indices to slots is valid as long as both operands use it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ac {

typedef __bf16 bf16_t;
typedef _Float16 f16_t;
typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef f16_t f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;
constexpr int kThreads = 256;      // 4 waves per workgroup
constexpr int kRowsPerWave = 32;   // one 32-row MFMA block per wave
constexpr int kChunk = 128;        // keys / map columns staged per LDS chunk
constexpr int kVtStride = kChunk + 4;  // elements per row of the transposed V tile

__device__ __forceinline__ f32x16 mfma_bf16(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma_f16(f16x8 a, f16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// Row of the 32 x 32 result that register v of lane-half kh holds.
__device__ __forceinline__ int mfma_row(int v, int kh) {
  return 8 * (v >> 2) + 4 * kh + (v & 3);
}

// A pointer that is the same in every lane, moved into scalar registers: loads through it can
// then take "scalar base + 32-bit lane offset" addresses instead of a 64-bit address per lane.
template <typename T>
__device__ __forceinline__ const T* uniform_ptr(const T* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  // (rebuilt as a GLOBAL pointer: the round trip through integers would otherwise leave a
  // generic one, and loads through it would be flat loads)
  typedef const T __attribute__((address_space(1))) * global_ptr;
  return (const T*)(global_ptr)(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 p = {(bf16_t)lo, (bf16_t)hi};  // round-to-nearest-even
  return __builtin_bit_cast(uint32_t, p);
}

// Permutation of the 16-byte pieces of a V row staged row-major in LDS for the transposing
// read (ds_read_b64_tr_b16): piece p of key row r sits at position p ^ v_piece_swizzle(r).  One
// such read instruction serves 32 lanes per LDS cycle: four consecutive keys x the two
// 16-column halves of a 32-column block x two pieces.  With the key in bits 2..3 of the piece
// index (D = 128; at D = 64 a row is half as long, so the key's lowest bit already selects the
// bank half and only its second bit enters) those 32 accesses fall on 32 different 8-byte bank
// pairs.  Unchanged by r + 4, so a copy that advances by whole multiples of four rows keeps one
// lane offset.
template <int D>
__host__ __device__ constexpr int v_piece_swizzle(int r) {
  return D == 128 ? 4 * (r & 3) : 4 * ((r >> 1) & 1);
}

// Permutation of the 16-byte pieces of a K row staged row-major and unpadded in LDS: piece p of
// key row r sits at position p ^ k_piece_swizzle(r), so that the 16-byte operand reads of 32
// consecutive rows spread over all banks (unchanged by r + 256 / (D / 8)).
template <int D>
__host__ __device__ constexpr int k_piece_swizzle(int r) {
  return D == 128 ? (r & 15) : ((r >> 1) & 7);
}

// Stage V[j0 .. j0+nj)[0..D) (row-major, row stride D) into LDS transposed:
// vt[d * kVtStride + j] = V[j0 + j][d].  All 256 threads take part.  Each task
// moves a 4 (rows) x 8 (d) block: four 16-byte global loads, an in-register
// transpose, eight 8-byte LDS stores.  nj is a multiple of 4.
template <int D>
__device__ __forceinline__ void stage_v_transposed(const bf16_t* __restrict__ Vsrc, int nj,
                                                   bf16_t* __restrict__ vt, int tid) {
  constexpr int DQ = D / 8;
  const int ntask = (nj >> 2) * DQ;
  for (int task = tid; task < ntask; task += kThreads) {
    const int dq = task % DQ;
    const int jq = task / DQ;
    const u32x4* src = reinterpret_cast<const u32x4*>(Vsrc + (size_t)(4 * jq) * D + 8 * dq);
    u32x4 r0 = src[0];
    u32x4 r1 = src[D / 8];
    u32x4 r2 = src[2 * (D / 8)];
    u32x4 r3 = src[3 * (D / 8)];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      // elements d = 8dq + 2p (low halves) and 8dq + 2p + 1 (high halves)
      u32x2 even, odd;
      even.x = __builtin_amdgcn_perm(r1[p], r0[p], 0x05040100u);
      even.y = __builtin_amdgcn_perm(r3[p], r2[p], 0x05040100u);
      odd.x = __builtin_amdgcn_perm(r1[p], r0[p], 0x07060302u);
      odd.y = __builtin_amdgcn_perm(r3[p], r2[p], 0x07060302u);
      *reinterpret_cast<u32x2*>(vt + (8 * dq + 2 * p) * kVtStride + 4 * jq) = even;
      *reinterpret_cast<u32x2*>(vt + (8 * dq + 2 * p + 1) * kVtStride + 4 * jq) = odd;
    }
  }
}

// Write one wave's 32 x D result tile (held transposed in MFMA result
// registers: acc[db][v] = out[row = lane % 32][d = 32 db + mfma_row(v, kh)])
// to global memory as bf16, through a wave-private LDS buffer so that the
// global stores are full 16-byte pieces of contiguous rows.
//   ost: wave-private LDS, 32 * (D + 4) elements;  dst: &out[row0][0], row stride D.
template <int D>
__device__ __forceinline__ void store_tile_bf16(const f32x16 (&acc)[D / 32], float mul,
                                                bf16_t* __restrict__ ost,
                                                bf16_t* __restrict__ dst, int lane) {
  constexpr int OS = D + 4;
  const int i = lane & 31, kh = lane >> 5;
#pragma unroll
  for (int db = 0; db < D / 32; ++db)
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      u32x2 w;
      w.x = pack_bf16(acc[db][4 * vq] * mul, acc[db][4 * vq + 1] * mul);
      w.y = pack_bf16(acc[db][4 * vq + 2] * mul, acc[db][4 * vq + 3] * mul);
      *reinterpret_cast<u32x2*>(ost + i * OS + 32 * db + 8 * vq + 4 * kh) = w;
    }
  // wave-private buffer: LDS operations of one wave execute in order, so only the compiler
  // has to be kept from moving the reads above the writes
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  constexpr int PIECES = 32 * D / 8;   // 16-byte pieces in the tile
#pragma unroll
  for (int it = 0; it < PIECES / kWave; ++it) {
    const int p = it * kWave + lane;
    const int row = p / (D / 8), c8 = p % (D / 8);
    const u32x2* s = reinterpret_cast<const u32x2*>(ost + row * OS + 8 * c8);
    u32x4 w;
    u32x2 a = s[0], b = s[1];
    w.x = a.x; w.y = a.y; w.z = b.x; w.w = b.y;
    // written once, not re-read by the writing kernel: streaming store
    __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(dst + (size_t)row * D + 8 * c8));
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// The same, for kernels whose big LDS tiles stay in use while results leave: the wave's 32 x D
// result goes out in 16-row x 64-column passes through a SMALL wave-private buffer
// (16 x kSmallOutStride elements = 2176 bytes); every global store still covers whole 128-byte
// lines.
constexpr int kSmallOutStride = 64 + 4;
template <int D>
__device__ __forceinline__ void store_tile_bf16_small(const f32x16 (&acc)[D / 32], float mul,
                                                      bf16_t* __restrict__ ost,
                                                      bf16_t* __restrict__ dst, int lane) {
  const int il = lane & 31, kh = lane >> 5;
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
            w.x = pack_bf16(t[4 * vq] * mul, t[4 * vq + 1] * mul);
            w.y = pack_bf16(t[4 * vq + 2] * mul, t[4 * vq + 3] * mul);
            *reinterpret_cast<u32x2*>(ost + (il & 15) * kSmallOutStride + 32 * dbp + 8 * vq + 4 * kh) = w;
          }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        const int p = it * kWave + lane;
        const int row = p >> 3, c8 = p & 7;
        const u32x2* sp = reinterpret_cast<const u32x2*>(ost + row * kSmallOutStride + 8 * c8);
        u32x2 lo = sp[0], hi = sp[1];
        __builtin_nontemporal_store(
            u32x4{lo.x, lo.y, hi.x, hi.y},
            reinterpret_cast<u32x4*>(dst + (size_t)(16 * rh + row) * D + 64 * dh + 8 * c8));
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
    }
}

}  // namespace ac
