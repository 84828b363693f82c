// The whole MoHGE layer for a decode-sized call (at most 32 tokens, bf16) as ONE launch on
// gfx950: router (sections 3.2.1 and 3.2.2 of the paper), permutation, both projections of the
// expert networks (section 3.1) and the gated combine (appendix, first equation).
//
// The grid holds one workgroup (4 waves) per piece of work, in this order of logical index:
//   route    partial logit sums: a wave owns 16 tokens x 16 router rows x 256 hidden elements
//            (fp32 matrix cores, folded into fp64 every 64 elements, as in the router kernels);
//   select   4 tokens per workgroup: adds the partial sums in slice order and runs the selection
//            of the router; the last of these workgroups to finish sorts the (token, slot) pairs by
//            expert (the small permutation kernel's code) and publishes `ready`;
//   up       one unit of the decode up projection (expert, 64 hidden units): waits for `ready`,
//            leaves at once if the expert has no token, else streams its weight rows and adds one
//            to the expert's counter;
//   down     one unit of the decode down projection (expert, 128 output features): waits for the
//            expert's counter to reach its number of up units, streams its weight rows, stores the
//            rows of y_perm, and adds one to the counter of every (token, 128-feature block) it
//            holds; the unit that completes such a counter (each token has K_e experts) computes that
//            piece of y = sum over slots of gate * y_perm row, in slot order.
// The arithmetic of every piece is that of the separate calls (same code, same order), so y is
// bit-identical to mohge_route (split form) -> mohge_permute -> mohge_expert_ffn -> mohge_combine
// whenever the logits of the two router forms round alike, and deterministic in any case.
//
// Order and progress.  A workgroup's logical index is a ticket drawn from a counter when it
// starts, so every workgroup with a smaller index has started before it.  Waits only ever point
// to smaller indices (select -> route, up -> select, down -> up), hence to workgroups that are
// running or done, whatever order the hardware starts workgroups in.  Every wait is bounded; if
// one expires the launch still drains (a workgroup that never saw `ready` skips its work rather
// than read unpublished indices), and the last workgroup to leave writes the status word and, on
// failure, overwrites y with NaN.
//
// Hand-over of data between workgroups: the producer's rows are stored at device scope (up and
// down units) or followed by a device-scope fence (router), every wave waits for its stores, a
// workgroup barrier follows, then one thread adds to the counter (release); the consumer polls
// the counter and performs an acquire before the workgroup reads.  Nothing reads a handed-over
// line in this launch before its counter is complete.
//
// The control words (ticket, counters) live at the start of the workspace.  They must be zero
// when the call starts; the last workgroup to leave clears them again, so a workspace zeroed once
// serves any number of calls in stream order.
#include <string.h>

#include "common.h"
#include "permute_small.h"
#include "route_select.h"
#include "skinny.h"

namespace mohge {

constexpr int kDecSlice = 256;          // hidden elements per route wave task
constexpr int kDecMaxT = 32;
constexpr int kDecSelTokens = 4;        // tokens per select workgroup (one per wave)
constexpr int kDecCtlHead = 16;         // ints before the per-expert counters
constexpr int kDecSpinLimit = 1 << 20;  // polls of about a microsecond
enum { kCtlTicket = 0, kCtlParts = 1, kCtlSelected = 2, kCtlReady = 3, kCtlExited = 4, kCtlFailed = 5 };

struct DecodeArgs {
  RouteArgs r;
  PermArgs p;
  SkinnyArgs up, dn;
  int* ctl;               // [kDecCtlHead] control words, then up_done[Ne], then tok_done[T * ncb]
  int* status;            // written at the end of every launch: 0 ok, bit 0 a wait expired, bit 1 the
                          //   control words were not zero at the start
  int n_ctl;              // ints of ctl
  int n_route, n_select, n_up, n_down;
  int TB, OT, NS;         // route wave tasks: token blocks x router-row tiles x slices of d
  int ncb;                // 128-feature blocks of a row of y
  const float* gates;
  uint16_t* y;
  int spin_limit;
};

__device__ __forceinline__ int ctl_load(const int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// failures are collected in a control word; the last workgroup to leave turns it into the status
__device__ __forceinline__ void set_failed(const DecodeArgs& a, int bit) {
  __hip_atomic_fetch_or(&a.ctl[kCtlFailed], bit, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void poison_y(const DecodeArgs& a) {
  const long long n = (long long)a.r.T * a.r.d / 2;
  for (long long i = threadIdx.x; i < n; i += blockDim.x) reinterpret_cast<uint32_t*>(a.y)[i] = 0x7FC07FC0u;
}

// Every thread of the workgroup calls it.  True once *ctr >= target; false if the bounded wait
// expired (the status word then says so; the caller skips whatever would read unpublished
// indices, and otherwise carries on so that the launch drains).
__device__ __forceinline__ bool wg_wait(const DecodeArgs& a, const int* ctr, int target, int* s_word) {
  __syncthreads();                      // (nobody still reads the word from an earlier use)
  if (threadIdx.x == 0) {
    int polls = 0, ok = 1;
    while (ctl_load(ctr) < target) {
      if (++polls > a.spin_limit) { ok = 0; set_failed(a, 1); break; }
      __builtin_amdgcn_s_sleep(32);
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    *s_word = ok;
  }
  __syncthreads();
  return *s_word != 0;
}

// Every thread calls it after its last store of handed-over data.
__device__ __forceinline__ void wg_signal(int* ctr) {
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

// True when expert e has rows and what was published about them can be used as indices: the
// rows lie inside [0, P), there are at most T of them, and they name pairs in [0, P).  Anything
// else would mean counters that were not zero at the start let a workgroup run ahead of the
// permutation; such a unit does nothing (and the failure word says so).  Every thread calls it.
__device__ __forceinline__ bool rows_valid(const DecodeArgs& a, int e, int* s_word) {
  const int row0 = a.p.offsets[e], cnt = a.p.offsets[e + 1] - row0;
  if (cnt == 0) return false;
  __syncthreads();
  if (threadIdx.x == 0) s_word[1] = 1;
  __syncthreads();
  bool ok = row0 >= 0 && cnt > 0 && cnt <= a.r.T && row0 + cnt <= a.p.P;
  if (ok && (int)threadIdx.x < cnt) {
    const int pr = a.p.perm[row0 + threadIdx.x];
    ok = pr >= 0 && pr < a.p.P;
  }
  if (!ok) s_word[1] = 0;
  __syncthreads();
  const bool all = s_word[1] != 0;
  if (!all && threadIdx.x == 0) set_failed(a, 2);
  return all;
}

// Wave task wt of the route role: partial logits of 16 tokens x 16 router rows over one slice of d.
__device__ __forceinline__ void decode_route_partial(const DecodeArgs& a, int wt, int lane) {
  const RouteArgs& r = a.r;
  const int rr = lane & 15, q = lane >> 4;
  const int tb = wt % a.TB, ot = (wt / a.TB) % a.OT, sl = wt / (a.TB * a.OT);
  int t = 16 * tb + rr, o = 16 * ot + rr;
  if (t > r.T - 1) t = r.T - 1;
  if (o > r.NO - 1) o = r.NO - 1;
  const uint16_t* xr = static_cast<const uint16_t*>(r.x) + (size_t)t * r.d;
  const float* wr = o < r.Ng ? r.wg + (size_t)o * r.d : r.we + (size_t)(o - r.Ng) * r.d;
  const int kbeg = sl * kDecSlice;
  const int kend = kbeg + kDecSlice < r.d ? kbeg + kDecSlice : r.d;
  double tot[4] = {0.0, 0.0, 0.0, 0.0};
  // lane (rr, q) loads 8 consecutive hidden elements of its token and of its router row at
  // 8q inside every 32-element step: matrix-core instruction j of the step multiplies element j of
  // every lane, so the step's 32 indices are covered once whatever their order
  for (int k = kbeg; k < kend; k += 64) {
    float xa[2][8], wb[2][8];
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      load8<true>(xr, (size_t)(k + 32 * s + 8 * q), xa[s]);
      load8<false>(wr, (size_t)(k + 32 * s + 8 * q), wb[s]);
    }
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(xa[s][j], wb[s][j], acc, 0, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) tot[i] += (double)acc[i];
  }
  // accumulator element i of lane (rr, q): token 4q + i, router row rr of the 16 x 16 tile
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int tt = 16 * tb + 4 * q + i, oo = 16 * ot + rr;
    if (tt < r.T && oo < r.NO) r.gpart[((size_t)sl * r.T + tt) * r.NO + oo] = tot[i];
  }
}

__global__ void __launch_bounds__(256) decode_layer_kernel(const DecodeArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_word[2];
  __shared__ int s_list[kDecMaxT];
  __shared__ int s_nlist;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int total = (int)gridDim.x;
  if (threadIdx.x == 0) {
    s_word[0] = __hip_atomic_fetch_add(&a.ctl[kCtlTicket], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_nlist = 0;
  }
  __syncthreads();
  const int id = s_word[0];
  __syncthreads();
  int* const up_done = a.ctl + kDecCtlHead;
  int* const tok_done = up_done + a.r.Ne;
  const int base_sel = a.n_route, base_up = base_sel + a.n_select, base_dn = base_up + a.n_up;

  if (id < 0 || id >= total) {
    // the control words were not zero when the launch started: this workgroup has no work it
    // could name.  Say so (directly as well, in case no workgroup turns out to be the last).
    if (threadIdx.x == 0) {
      set_failed(a, 2);
      __hip_atomic_store(a.status, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (blockIdx.x == 0) poison_y(a);
  } else if (id < base_sel) {
    // ---- route: partial logit sums ----------------------------------------------------------
    const int wt = id * 4 + w;
    if (wt < a.TB * a.OT * a.NS) decode_route_partial(a, wt, lane);
    wg_signal(&a.ctl[kCtlParts]);
  } else if (id < base_up) {
    // ---- select: logits of 4 tokens, selection; the last one sorts the pairs -----------------
    const int t0 = (id - base_sel) * kDecSelTokens;
    wg_wait(a, &a.ctl[kCtlParts], a.n_route, &s_word[1]);
    float* lg = reinterpret_cast<float*>(smem + a.r.region0);       // [4][NOpad]
    for (int idx = threadIdx.x; idx < kDecSelTokens * a.r.NO; idx += blockDim.x) {
      const int tl = idx / a.r.NO, o = idx % a.r.NO;
      double sum = 0.0;
      if (t0 + tl < a.r.T)
        for (int sp = 0; sp < a.NS; ++sp) sum += a.r.gpart[((size_t)sp * a.r.T + t0 + tl) * a.r.NO + o];
      lg[tl * a.r.NOpad + o] = (float)sum;
    }
    __syncthreads();
    route_select(a.r, smem, lg, t0, kDecSelTokens, 4, w, lane);
    __threadfence();
    __syncthreads();
    if (threadIdx.x == 0)
      s_word[1] = __hip_atomic_fetch_add(&a.ctl[kCtlSelected], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (s_word[1] == a.n_select - 1) {
      // every token's experts are in place (and visible: the acquire above): stable counting sort
      int(*hist)[kMaxExperts] = reinterpret_cast<int(*)[kMaxExperts]>(smem);
      int* wtot = reinterpret_cast<int*>(smem + sizeof(int) * kWavesPerBlock * kMaxExperts);
      permute_small_body(a.p, hist, wtot);
      wg_signal(&a.ctl[kCtlReady]);
    }
  } else if (id < base_dn) {
    // ---- up unit ------------------------------------------------------------------------------
    const int blk = id - base_up;
    const bool ready = wg_wait(a, &a.ctl[kCtlReady], 1, &s_word[1]);
    int g = 0;
    while (g + 1 < a.up.Ng && blk >= a.up.blk_prefix[g + 1]) ++g;
    const int e = g * a.up.N + (blk - a.up.blk_prefix[g]) / (a.up.F[g] / 64);
    if (ready && rows_valid(a, e, s_word)) {
      skinny_unit<true, true>(a.up, blk);
      wg_signal(&up_done[e]);
    }
  } else {
    // ---- down unit, and the pieces of y it completes --------------------------------------------
    const int blk = id - base_dn;
    const bool ready = wg_wait(a, &a.ctl[kCtlReady], 1, &s_word[1]);
    int g = 0;
    while (g + 1 < a.dn.Ng && blk >= a.dn.blk_prefix[g + 1]) ++g;
    const int local = blk - a.dn.blk_prefix[g];
    const int e = g * a.dn.N + local / a.ncb, cb = local % a.ncb;
    const bool live = ready && rows_valid(a, e, s_word);
    const int row0 = live ? a.dn.offsets[e] : 0, cnt = live ? a.dn.offsets[e + 1] - row0 : 0;
    if (cnt > 0) {
      wg_wait(a, &up_done[e], a.dn.F[g] / 64, &s_word[1]);
      skinny_unit<false, true>(a.dn, blk);
      __threadfence();
      __syncthreads();
      // one thread per routed row of the expert: its token's counter for this feature block
      for (int tt = threadIdx.x; tt < cnt; tt += blockDim.x) {
        const int t = a.p.perm[row0 + tt] / a.dn.Ke;
        const int old = __hip_atomic_fetch_add(&tok_done[t * a.ncb + cb], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        if (old == a.dn.Ke - 1) {
          const int at = atomicAdd(&s_nlist, 1);
          if (at < kDecMaxT) s_list[at] = t;
        }
      }
      __syncthreads();
      // y[t, 128 features] for the listed tokens: 16 bytes per thread, fp32 accumulation in slot
      // order (the arithmetic of the combine kernel)
      const int nl = s_nlist < kDecMaxT ? s_nlist : kDecMaxT;
      const uint4* yp = reinterpret_cast<const uint4*>(a.dn.C);
      const int vec_per_row = a.dn.d / 8;
      for (int i = threadIdx.x; i < nl * 16; i += blockDim.x) {
        const int t = s_list[i >> 4], v = cb * 16 + (i & 15);
        if (v >= vec_per_row) continue;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int slot = 0; slot < a.dn.Ke; ++slot) {
          const float gt = a.gates[(size_t)t * a.dn.Ke + slot];
          int rw = a.p.inv_perm[(size_t)t * a.dn.Ke + slot];
          rw = rw < 0 ? 0 : (rw >= a.p.P ? a.p.P - 1 : rw);     // (never outside y_perm, whatever was published)
          const uint4 u = yp[(size_t)rw * vec_per_row + v];
          acc[0] = fmaf(gt, __uint_as_float(u.x << 16), acc[0]);
          acc[1] = fmaf(gt, __uint_as_float(u.x & 0xffff0000u), acc[1]);
          acc[2] = fmaf(gt, __uint_as_float(u.y << 16), acc[2]);
          acc[3] = fmaf(gt, __uint_as_float(u.y & 0xffff0000u), acc[3]);
          acc[4] = fmaf(gt, __uint_as_float(u.z << 16), acc[4]);
          acc[5] = fmaf(gt, __uint_as_float(u.z & 0xffff0000u), acc[5]);
          acc[6] = fmaf(gt, __uint_as_float(u.w << 16), acc[6]);
          acc[7] = fmaf(gt, __uint_as_float(u.w & 0xffff0000u), acc[7]);
        }
        uint4 o;
        o.x = pack_bf16x2(acc[0], acc[1]);
        o.y = pack_bf16x2(acc[2], acc[3]);
        o.z = pack_bf16x2(acc[4], acc[5]);
        o.w = pack_bf16x2(acc[6], acc[7]);
        reinterpret_cast<uint4*>(a.y)[(size_t)t * vec_per_row + v] = o;
      }
    }
  }

  // ---- the last workgroup to leave clears the control words for the next call -------------------
  __syncthreads();
  if (threadIdx.x == 0)
    s_word[1] = __hip_atomic_fetch_add(&a.ctl[kCtlExited], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
  __syncthreads();
  if (s_word[1] == total - 1) {
    const int failed = ctl_load(&a.ctl[kCtlFailed]);
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(a.status, failed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int i = threadIdx.x; i < a.n_ctl; i += blockDim.x) a.ctl[i] = 0;
    if (failed) poison_y(a);
  }
}

// ---- host ------------------------------------------------------------------------------------------
struct DecodeLayout {
  size_t ctl, status, gpart, counts, offsets, perm, inv_perm, h, y_perm, total;
  int n_ctl, ncb, NS;
};

static DecodeLayout decode_layout(const LayerDesc& L) {
  DecodeLayout o;
  auto up256 = [](size_t b) { return (b + 255) / 256 * 256; };
  o.ncb = (L.d + 127) / 128;
  o.NS = (L.d + kDecSlice - 1) / kDecSlice;
  o.n_ctl = kDecCtlHead + L.Ne + L.T * o.ncb;
  size_t at = 0;
  o.ctl = at; at += up256((size_t)o.n_ctl * sizeof(int));
  o.status = at; at += 256;
  o.gpart = at; at += up256((size_t)o.NS * L.T * (L.Ng + L.Ne) * sizeof(double));
  o.counts = at; at += up256((size_t)L.Ne * sizeof(int));
  o.offsets = at; at += up256((size_t)(L.Ne + 1) * sizeof(int));
  o.perm = at; at += up256((size_t)L.P * sizeof(int));
  o.inv_perm = at; at += up256((size_t)L.P * sizeof(int));
  o.h = at; at += up256((size_t)L.P * L.Fmax * 2);
  o.y_perm = at; at += up256((size_t)L.P * L.d * 2);
  o.total = at;
  return o;
}

bool decode_layer_supported(const LayerDesc& L, int dtype) {
  return dtype == MOHGE_BF16 && L.T <= kDecMaxT && L.P <= kBlockPairs;
}

size_t decode_layer_workspace_bytes(const LayerDesc& L) {
  LayerDesc M = L;
  if (M.T < 1) { M.T = 1; M.P = M.Ke; }
  return decode_layout(M).total;
}

size_t decode_layer_ctl_bytes(const LayerDesc& L) {
  LayerDesc M = L;
  if (M.T < 1) { M.T = 1; M.P = M.Ke; }
  return decode_layout(M).status;       // (the status word follows the control words)
}

hipError_t launch_decode_layer(const LayerDesc& L, const void* x, const float* w_group, const float* w_expert,
                               const float* bias, const GroupPtrs& W, int32_t* group_idx, int32_t* expert_idx,
                               float* gates, void* y, void* ws, int spin_limit, hipStream_t s) {
  const DecodeLayout lay = decode_layout(L);
  unsigned char* base = static_cast<unsigned char*>(ws);
  DecodeArgs a;
  memset(&a, 0, sizeof(a));
  RouteArgs& r = a.r;
  r.x = x; r.wg = w_group; r.we = w_expert; r.bias = bias;
  r.gidx = group_idx; r.eidx = expert_idx; r.gates = gates; r.gs = nullptr; r.es1 = nullptr;
  r.T = L.T; r.d = L.d; r.Ng = L.Ng; r.N = L.N; r.Ne = L.Ne; r.Kg = L.Kg; r.Ke = L.Ke;
  r.mode = L.select_mode;
  r.NO = L.Ng + L.Ne;
  r.NOpad = ((r.NO + 15) / 16) * 16 + 4;
  r.Nepad = ((L.Ne + 63) / 64) * 64;
  r.kslice = kDecSlice;
  r.region0 = (int)(((size_t)4 * 5 * r.Nepad * sizeof(float) + 15) / 16 * 16);
  r.dsplit = lay.NS;
  r.gpart = reinterpret_cast<double*>(base + lay.gpart);
  PermArgs& p = a.p;
  p.eidx = expert_idx;
  p.counts = reinterpret_cast<int32_t*>(base + lay.counts);
  p.offsets = reinterpret_cast<int32_t*>(base + lay.offsets);
  p.perm = reinterpret_cast<int32_t*>(base + lay.perm);
  p.inv_perm = reinterpret_cast<int32_t*>(base + lay.inv_perm);
  p.seg_hist = nullptr;
  p.P = L.P; p.Ne = L.Ne; p.nseg = (L.P + kSegPairs - 1) / kSegPairs;
  p.nbits = 0;
  while ((1 << p.nbits) < L.Ne) ++p.nbits;
  int nu = 0, nd = 0;
  skinny_args(L, x, p.perm, p.offsets, W, base + lay.y_perm, base + lay.h, nullptr, nullptr, nullptr, nullptr,
              a.up, a.dn, nu, nd);
  a.ctl = reinterpret_cast<int*>(base + lay.ctl);
  a.status = reinterpret_cast<int*>(base + lay.status);
  a.n_ctl = lay.n_ctl;
  a.TB = (L.T + 15) / 16;
  a.OT = (r.NO + 15) / 16;
  a.NS = lay.NS;
  a.n_route = (a.TB * a.OT * a.NS + 3) / 4;
  a.n_select = (L.T + kDecSelTokens - 1) / kDecSelTokens;
  a.n_up = nu;
  a.n_down = nd;
  a.ncb = lay.ncb;
  a.gates = gates;
  a.y = static_cast<uint16_t*>(y);
  a.spin_limit = spin_limit == 0 ? kDecSpinLimit : spin_limit;
  const size_t sel = (size_t)r.region0 + (size_t)kDecSelTokens * r.NOpad * sizeof(float);
  const size_t srt = sizeof(int) * (kWavesPerBlock * kMaxExperts + kWavesPerBlock);
  const size_t smem = sel > srt ? sel : srt;
  const unsigned grid = (unsigned)(a.n_route + a.n_select + a.n_up + a.n_down);
  hipLaunchKernelGGL(decode_layer_kernel, dim3(grid), dim3(256), smem, s, a);
  return hipGetLastError();
}

long long decode_layer_status_offset(const LayerDesc& L) { return (long long)decode_layout(L).status; }

}  // namespace mohge
