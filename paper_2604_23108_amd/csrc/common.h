// Internal declarations shared by the host entry points and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mohge.h"

namespace mohge {

constexpr int kMaxGroups = 16;
constexpr int kMaxExperts = 256;
constexpr int kWave = 64;

// Layer description passed by value to kernels (everything a kernel needs to map an
// expert id to its group, width and weight block).
struct LayerDesc {
  int32_t T, d, Ng, N, Ne, Kg, Ke, P;
  int32_t select_mode;
  int32_t F[kMaxGroups];          // F_g
  int32_t Fmax;
};

struct GroupPtrs {
  const void* w13[kMaxGroups];    // [N, 2F_g, d]
  const void* w2[kMaxGroups];     // [N, d, F_g]
};

// How the matrix-core path of the expert networks is launched.  The entry points of mohge.h use
// the defaults; the benchmark library passes its caller's choices.  Results do not depend on any
// of these (except a negative spin_limit, a test hook).
struct FfnOptions {
  int tile_rows[2] = {0, 0};  // token-tile height of the up / down list: 0 = chosen per call, else 64..256
  int fused = 1;              // both projections (dH and dX; the two weight gradients) in one launch
  int spin_limit = 0;         // polls a dependent tile waits: 0 = default (about a second), < 0 = give up at once
  int band = 4;               // row blocks per band of the tile order inside an expert
  int group_major = 0;        // 1: experts visited group by group, 0: by all-size sets
  int steal = 2;              // workgroups whose XCD range is exhausted help the other ranges: bit 0 in the first
                              //   list of a fused launch, bit 1 in the second
  int short_last = 1;         // second list of a fused launch: the tiles with the shortest reduction last in every XCD range
  int defer_signal = 1;       // first list of a fused launch: a finished tile is announced once the workgroup's next tile
                              //   has its first stage (whose arrival proves the stores complete) instead of after a wait
  long long* cycles = nullptr;  // DEVICE, optional: per-workgroup clock counters of the fused launch
  int cycles_launch = 0;      // backward: which of the two fused launches fills `cycles` (0 = dH/dX, 1 = weight gradients)
};

void set_error(const char* fmt, ...);
int check_config(const mohge_config* cfg, LayerDesc* out);
// pointer check shared by the entry points: NULL (when required) and 16-byte alignment
int need(const void* p, const char* name, bool required);
int hip_rc(hipError_t e, const char* what);

// bf16 <-> fp32 on the device, bit level (round to nearest even on the way down)
__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
// two floats -> packed bf16 pair with the hardware conversion (v_cvt_pk_bf16_f32, round
// to nearest even); `lo` lands in the low half
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  const bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
  return __builtin_bit_cast(uint32_t, r);
}
// SiLU(g) * u with the fast exp / reciprocal instructions (relative error ~1e-6, far
// below the bf16 rounding that follows)
__device__ __forceinline__ float swiglu(float g, float u) {
  return g * u * __builtin_amdgcn_rcpf(1.f + __expf(-g));
}

// launchers implemented in the kernel files; each returns a hipError_t from the launch
hipError_t launch_route(const LayerDesc& L, int dtype, const void* x, const float* w_group,
                        const float* w_expert, const float* bias, int32_t* group_idx,
                        int32_t* expert_idx, float* gates, float* gs_out, float* es1_out,
                        void* ws, size_t ws_bytes, hipStream_t s);
size_t route_workspace_bytes(const LayerDesc& L, int dtype);
bool ffn_w8_supported(const LayerDesc& L);
hipError_t launch_expert_ffn_w8(const LayerDesc& L, const void* x, const int32_t* perm,
                                const int32_t* offsets, const GroupPtrs& Wq, const float* const* s13,
                                const float* const* s2, void* y_perm, void* ws, hipStream_t s);
hipError_t launch_fp8_decode(const void* q, float* out, long long n, hipStream_t s);
hipError_t launch_expert_ffn_w4(const LayerDesc& L, const void* x, const int32_t* perm,
                                const int32_t* offsets, const GroupPtrs& Wq, const void* const* b13,
                                const void* const* b2, void* y_perm, void* ws, hipStream_t s);
hipError_t launch_mxfp4_decode(const void* packed, const void* scales, float* out, long long n, hipStream_t s);
size_t permute_workspace_bytes(const LayerDesc& L);
hipError_t launch_permute(const LayerDesc& L, int dtype, const int32_t* expert_idx,
                          int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                          const void* x, void* x_perm, void* ws, hipStream_t s);
hipError_t launch_permute_static(const LayerDesc& L, int dtype, const int32_t* expert_idx,
                                 int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                                 const void* x, void* x_perm, hipStream_t s);
size_t ffn_workspace_bytes(const LayerDesc& L, int dtype);
hipError_t launch_expert_ffn(const LayerDesc& L, int dtype, const void* x, const int32_t* perm,
                             const int32_t* offsets, const GroupPtrs& W, void* y_perm, void* ws,
                             hipStream_t s, int stages, int parts = 3,
                             const FfnOptions& o = FfnOptions());   // stages: bit 0 = up, bit 1 = down
bool ffn_parts_supported(const LayerDesc& L, int dtype);
// byte offset of the schedule header that carries the "gave up waiting" flag of a fused launch in
// the workspace of call `which_call`, or -1 where the call has no fused launch
long long fused_flag_offset(const LayerDesc& L, int dtype, int which_call);
hipError_t launch_combine(const LayerDesc& L, int dtype, const void* y_perm,
                          const int32_t* inv_perm, const float* gates, const void* y_add, void* y,
                          hipStream_t s);
hipError_t launch_shared_routing(const LayerDesc& L, int32_t* expert_idx, float* gates,
                                 int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                                 hipStream_t s);
// training: forward that keeps what the backward pass needs, and the backward launchers (bf16)
size_t ffn_saved_bytes(const LayerDesc& L);
hipError_t launch_expert_ffn_train(const LayerDesc& L, const void* x, const int32_t* perm,
                                   const int32_t* offsets, const GroupPtrs& W, void* y_perm,
                                   void* saved, hipStream_t s, const FfnOptions& o = FfnOptions());
hipError_t launch_combine_bwd(const LayerDesc& L, const void* dy, const void* y_perm,
                              const int32_t* inv_perm, const float* gates, float* dgates,
                              void* dy_perm, hipStream_t s);
size_t ffn_bwd_workspace_bytes(const LayerDesc& L);
hipError_t launch_expert_ffn_bwd(const LayerDesc& L, const void* x, const int32_t* perm,
                                 const int32_t* offsets, const GroupPtrs& W, const void* saved,
                                 const void* dy_perm, void* dx_perm, void* const* dw13,
                                 void* const* dw2, void* ws, hipStream_t s,
                                 const FfnOptions& o = FfnOptions());
size_t route_bwd_workspace_bytes(const LayerDesc& L);
hipError_t launch_route_bwd(const LayerDesc& L, const mohge_config& cfg, const void* x,
                            const float* w_group, const float* w_expert, const float* gs,
                            const float* es1, const int32_t* group_idx, const int32_t* expert_idx,
                            const float* gates, const float* dgates, const float* stats,
                            const void* dx_perm, const int32_t* inv_perm, void* dx, float* dw_group,
                            float* dw_expert, float* dz_out, void* ws, hipStream_t s);
size_t tiled_sched_bytes(const LayerDesc& L);
// the whole layer of a decode-sized call in one launch (decode_layer.hip)
bool decode_layer_supported(const LayerDesc& L, int dtype);
size_t decode_layer_workspace_bytes(const LayerDesc& L);
size_t decode_layer_ctl_bytes(const LayerDesc& L);
long long decode_layer_status_offset(const LayerDesc& L);
long long decode_layer_trace_entries(const LayerDesc& L);
hipError_t launch_decode_layer(const LayerDesc& L, const void* x, const float* w_group, const float* w_expert,
                               const float* bias, const GroupPtrs& W, int32_t* group_idx, int32_t* expert_idx,
                               float* gates, void* y, void* ws, int spin_limit, long long* trace, hipStream_t s);
size_t aux_workspace_bytes(const LayerDesc& L);
hipError_t launch_aux_loss(const LayerDesc& L, const mohge_config& cfg, const float* gs,
                           const float* es1, const int32_t* group_idx, const int32_t* expert_idx,
                           float* losses, float* stats, void* ws, hipStream_t s);

}  // namespace mohge
