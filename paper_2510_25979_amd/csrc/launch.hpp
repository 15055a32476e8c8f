// Host-side launch descriptors shared by the C-ABI layer (api.hip) and the
// kernel files.  Everything here is plain data; validation happens in api.hip
// before a descriptor is filled.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

namespace ac {

// Dynamic LDS above 64 KiB needs a per-kernel opt-in; done once per kernel and size.
template <auto Kernel>
inline hipError_t ensure_lds(size_t bytes) {
  // Host threads may launch the same kernel at once: the largest size granted so far is an
  // atomic that only grows; two threads that both see it too small both set the attribute
  // (the larger request wins in the maximum, and setting it twice is harmless).
  static std::atomic<size_t> granted{64 * 1024};
  if (bytes <= granted.load(std::memory_order_acquire)) return hipSuccess;
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kernel),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e != hipSuccess) return e;
  size_t seen = granted.load(std::memory_order_relaxed);
  while (seen < bytes && !granted.compare_exchange_weak(seen, bytes, std::memory_order_release)) {}
  return e;
}

struct ApplyLaunch {
  const void* maps;      // device: whole database, or a single staged entry (fixed_entry >= 0)
  const int32_t* hit;    // device [B]; unused when fixed_entry >= 0
  const void* V;
  void* O;
  int32_t B, M, L, layer_begin, Lc, Hq, Hkv, S, D;
  int32_t causal, is_f32;
  int32_t packed;        // bf16 only: maps are stored in the packed block layout
  int32_t fixed_entry;   // -1: index through hit[]
  int32_t n_list;        // queries in q_list (<= 32) when fixed_entry >= 0
  int32_t q_list[32];
};
hipError_t launch_apply(const ApplyLaunch& p, hipStream_t stream);
hipError_t launch_pack_maps(const void* dense, void* packed, int64_t n_tiles, int32_t S,
                            int32_t causal, hipStream_t stream);

// Packed map layout: 16-row block r keeps its first packed_cols(r) blocks of 32 columns
// (causal: ceil((r+1)/2); dense: all S/32), 512 elements each, row-block-major.
__host__ __device__ inline int packed_prefix(int r) { return ((r + 1) >> 1) * ((r + 2) >> 1); }
__host__ __device__ inline int packed_blocks(int S, int causal) {
  return causal ? packed_prefix(S >> 4) : (S >> 4) * (S >> 5);
}

struct ExactLaunch {
  const void *Q, *K, *V;
  void* O;
  const int32_t* row_sel;
  const int32_t* key_len;   // device [B] or nullptr
  int32_t B, Hq, Hkv, S, D, causal, is_f32;
  float scale;
};
hipError_t launch_exact(const ExactLaunch& p, hipStream_t stream);

struct InsertLaunch {
  const void *Q, *K, *V;   // device [B][Lc][Hq|Hkv][S][D] bf16
  void* O;                 // device [B][Lc][Hq][S][D] bf16
  void* maps;              // device: the whole map store (bf16, dense or packed)
  const void* feat;        // device [B][E] or nullptr (maps only)
  void* emb;               // device: the whole feature store
  const int32_t* slot;     // device [B] or nullptr (compute O only)
  const int32_t* row_sel;  // device [B] or nullptr
  const int32_t* key_len;  // device [B] or nullptr
  int32_t B, M, L, layer_begin, Lc, Hq, Hkv, S, D, causal, packed;
  int32_t emb_row_bytes;
  float scale;
};
hipError_t launch_insert(const InsertLaunch& p, hipStream_t stream);

struct SearchLaunch {
  const void* emb;        // device [N][E]
  const void* q;          // device [B][E]
  const int32_t* map_of;  // device [N] or nullptr
  int32_t N, E, B, k, is_f16, metric;
  float threshold;
  int32_t *idx, *hit;
  float* score;
  void* ws;
  size_t ws_bytes;
};
size_t search_workspace_bytes(int32_t N, int32_t E, int32_t B, int32_t k, int32_t is_f16);
hipError_t launch_search(const SearchLaunch& p, hipStream_t stream);

struct ProjectLaunch {
  const void* h;            // device [B][S][dm], bf16 or fp32
  const int32_t* seq_len;   // device [B] or nullptr
  const float *W1, *b1;     // device [hid][dm], [hid] or nullptr
  const float *W2, *b2;     // device [E][hid], [E] or nullptr
  void* feat;               // device [B][E], fp16 or fp32
  void* ws;
  int32_t B, S, dm, hid, E, h_is_f32, feat_is_f16, normalize;
};
size_t project_workspace_bytes(int32_t B, int32_t dm, int32_t hid, int32_t E);
hipError_t launch_project(const ProjectLaunch& p, hipStream_t stream);

}  // namespace ac
