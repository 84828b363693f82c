// The whole MoHGE layer for a decode-sized call (at most 32 tokens, bf16) as ONE launch on
// gfx950: router (sections 3.2.1 and 3.2.2 of the paper), permutation, both projections of the
// expert networks (section 3.1) and the gated combine (appendix, first equation).
//
// Persistent workgroups (4 waves; as many as the device holds at once) draw pieces of work from
// two counters, each in dependency order:
//  first queue   route tasks, then select tasks.  A route task is the partial logits of 16
//                tokens x 16 router rows over 256 hidden elements (fp32 matrix cores, 64 elements
//                per wave, the waves' sums and everything after them in fp64, as in the router
//                kernels).  A select task adds the partial sums of 4 tokens in slice order and runs
//                the router's selection; the last one to finish sorts the (token, slot) pairs by
//                expert (the small permutation kernel's code) and publishes `ready`.
//  second queue  every workgroup waits for `ready`, reads `offsets` and numbers the units of the
//                experts that have rows.  Up units first (expert, 64 hidden units: the decode up
//                projection's unit), expert by expert; the unit that completes an expert appends it
//                to a list.  Then down units (expert, 128 output features), taking the experts in
//                the order of that list, so that a unit waits only when no expert at all is ready.
//                A down unit stores its rows of y_perm and adds one to the counter of every
//                (token, 128-feature block) it holds; the unit that completes such a counter (each
//                token has K_e experts) computes that piece of y = sum over slots of gate * y_perm
//                row, in slot order.
// The arithmetic of every piece is that of the separate calls (same code, same order), so given
// the routing y is bit-identical to mohge_permute -> mohge_expert_ffn -> mohge_combine, and the
// routing is that of mohge_route up to the grouping of the fp64 partial sums.
//
// Progress.  Work is drawn in an order in which everything a piece waits for was drawn earlier
// (select after route, down after up), so it is in the hands of a running workgroup that never
// waits itself for anything later: no assumption about how many workgroups are resident or in
// which order the hardware starts them.  (A workgroup requests its next draw while it works; the
// unit it holds back that way is always later in the queue than the one in hand.)  Every wait is
// bounded; if one expires the launch still drains (a workgroup that never saw `ready` takes no
// units rather than read unpublished indices), and the last workgroup to leave writes the status
// word and, on failure, overwrites y with NaN.
//
// Hand-over of data between workgroups: the producer's rows are stored at device scope, i.e.
// written through the XCD's L2 (route partial sums, H, y_perm), or followed by a device-scope
// fence (the selection's outputs and the permutation: a handful of workgroups; that fence walks
// the whole L2, one per unit cost a millisecond); every wave waits for its stores, a workgroup
// barrier follows, then one thread adds to the counter; the consumer polls the counter at device
// scope.  Nothing reads a handed-over line in this launch before its counter is complete, and
// launch boundaries invalidate the caches, so no cache can hold an older copy.  Waiting
// workgroups poll memory every few microseconds, and the list entries they poll are 256 bytes
// apart: polls of one line by hundreds of workgroups were a hot spot in one memory channel that
// slowed the weight streams of everybody else.
//
// The control words (queue counters, per-expert and per-token counters, the list) live at the
// start of the workspace.  They must be zero when the call starts; the last workgroup to leave
// clears them again, so a workspace zeroed once serves any number of calls in stream order.
#include <string.h>

#include "common.h"
#include "permute_small.h"
#include "route_select.h"
#include "skinny.h"

namespace mohge {

constexpr int kDecSlice = 64;           // hidden elements per route wave task
constexpr int kDecMaxT = 32;
constexpr int kDecSelTokens = 4;        // tokens per select workgroup (one per wave)
constexpr int kDecCtlHead = 16;         // ints before the per-expert counters
constexpr int kDoneStride = 64;         // ints between entries of the completed-expert list: the workgroups that wait
                                        // for an entry poll it in memory, and entries 256 bytes apart sit in
                                        // different memory channels instead of all polls hitting one
constexpr int kDecSpinLimit = 1 << 19;  // polls a microsecond or a few apart
enum { kCtlNextA = 0, kCtlParts = 1, kCtlSelected = 2, kCtlReady = 3, kCtlExited = 4, kCtlFailed = 5, kCtlNextB = 6, kCtlDoneTail = 7 };

struct DecodeArgs {
  RouteArgs r;
  PermArgs p;
  SkinnyArgs up, dn;
  int* ctl;               // [kDecCtlHead] control words, then up_done[Ne], done_list[Ne], tok_done[T * ncb]
  int* status;            // written at the end of every launch: 0 ok, bit 0 a wait expired, bit 1 the
                          //   control words were not zero at the start
  int n_ctl;              // ints of ctl
  int n_route, n_select, n_up, n_down;
  int TB, OT, NS, NSP;    // route tasks: token blocks x router-row tiles x NS slices of d (256 elements);
                          //   NSP: NS rounded up to even, the partial sums of a logit in memory
  int ncb;                // 128-feature blocks of a row of y
  const float* gates;
  uint16_t* y;
  int spin_limit;
  long long* trace;       // NULL, or [workgroups][4] 100 MHz time stamps by logical index: start, after the wait for
                          //   `ready` (or the route partials), after the wait for the expert's up units, end
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

// Every thread calls it.  The value of *p once it is not zero, or 0 if the bounded wait expired.
__device__ __forceinline__ int wg_wait_value(const DecodeArgs& a, const int* p, int* s_word) {
  __syncthreads();
  if (threadIdx.x == 0) {
    int polls = 0, v;
    while ((v = ctl_load(p)) == 0) {
      if (++polls > a.spin_limit) { set_failed(a, 1); break; }
      __builtin_amdgcn_s_sleep(127);
    }
    *s_word = v;
  }
  __syncthreads();
  return *s_word;
}

// Every thread calls it after its last store of handed-over data.  WRITTEN_THROUGH: all of that
// data was stored at device scope (store*_device_scope), so waiting for the stores is enough;
// otherwise a device-scope fence writes the XCD's L2 back first.  That fence walks the whole
// cache: a few dozen of them per launch are free, one per unit is not (measured: 3400 of them
// turned a 0.38 ms step into 1.36 ms).
template <bool WRITTEN_THROUGH>
__device__ __forceinline__ void wg_signal(int* ctr) {
  if constexpr (WRITTEN_THROUGH) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  else __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Route task: partial logits of 16 tokens x 16 router rows over 256 hidden elements, 64 per wave
// (one round trip to memory), the four waves' fp64 sums added through LDS in wave order.
__device__ __forceinline__ void decode_route_partial(const DecodeArgs& a, int task, unsigned char* smem, int lane, int w) {
  const RouteArgs& r = a.r;
  const int rr = lane & 15, q = lane >> 4;
  const int tb = task % a.TB, ot = (task / a.TB) % a.OT, sg = task / (a.TB * a.OT);
  int t = 16 * tb + rr, o = 16 * ot + rr;
  if (t > r.T - 1) t = r.T - 1;
  if (o > r.NO - 1) o = r.NO - 1;
  const uint16_t* xr = static_cast<const uint16_t*>(r.x) + (size_t)t * r.d;
  const float* wr = o < r.Ng ? r.wg + (size_t)o * r.d : r.we + (size_t)(o - r.Ng) * r.d;
  const int k = (4 * sg + w) * kDecSlice;
  double tot[4] = {0.0, 0.0, 0.0, 0.0};
  if (k < r.d) {
    // lane (rr, q) loads 8 consecutive hidden elements of its token and of its router row at
    // 8q inside both 32-element steps: matrix-core instruction j of a step multiplies element j
    // of every lane, so the step's 32 indices are covered once whatever their order
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
    for (int i = 0; i < 4; ++i) tot[i] = (double)acc[i];
  }
  // accumulator element i of lane (rr, q): token 4q + i, router row rr of the 16 x 16 tile
  double* part = reinterpret_cast<double*>(smem);                 // [4 waves][16 tokens][16 rows]
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 4; ++i) part[(w * 16 + 4 * q + i) * 16 + rr] = tot[i];
  __syncthreads();
  {
    const int tl = threadIdx.x >> 4, ol = threadIdx.x & 15;
    const double sum = ((part[threadIdx.x] + part[256 + threadIdx.x]) + part[512 + threadIdx.x]) + part[768 + threadIdx.x];
    const int tt = 16 * tb + tl, oo = 16 * ot + ol;
    // written through (a consumer on another XCD reads it in this launch)
    if (tt < r.T && oo < r.NO) {
      const unsigned long long bits = __double_as_longlong(sum);
      store8_device_scope(r.gpart + ((size_t)tt * r.NO + oo) * a.NSP + sg, make_uint2((unsigned)bits, (unsigned)(bits >> 32)));
    }
  }
}

// Broadcast of one int from thread 0 to the workgroup through an LDS word.
__device__ __forceinline__ int wg_bcast(int v, int* word) {
  __syncthreads();                      // (nobody still reads the word from an earlier use)
  if (threadIdx.x == 0) *word = v;
  __syncthreads();
  return *word;
}

__device__ __forceinline__ int draw(int* ctr) {
  return __hip_atomic_fetch_add(ctr, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Select task: 4 tokens; the last task to finish sorts the pairs and publishes `ready`.
__device__ __forceinline__ void decode_select(const DecodeArgs& a, int task, unsigned char* smem, int* s_word,
                                              int lane, int w) {
  const int t0 = task * kDecSelTokens;
  wg_wait(a, &a.ctl[kCtlParts], a.n_route, &s_word[1]);
  float* lg = reinterpret_cast<float*>(smem + a.r.region0);       // [4][NOpad]
  for (int idx = threadIdx.x; idx < kDecSelTokens * a.r.NO; idx += blockDim.x) {
    const int tl = idx / a.r.NO, o = idx % a.r.NO;
    double sum = 0.0;
    if (t0 + tl < a.r.T) {
      // the NS partial sums of a logit are neighbours in memory: loaded two at a time, all requests
      // before the first addition, added in slice order
      const double2* gp = reinterpret_cast<const double2*>(a.r.gpart + ((size_t)(t0 + tl) * a.r.NO + o) * a.NSP);
      for (int sp = 0; sp < a.NS; sp += 16) {
        double2 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          v[u] = sp + 2 * u < a.NS ? gp[sp / 2 + u] : make_double2(0.0, 0.0);
          if (sp + 2 * u + 1 >= a.NS) v[u].y = 0.0;              // (the padding slot of an odd count)
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) { sum += v[u].x; sum += v[u].y; }
      }
    }
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
    __syncthreads();
    permute_small_body(a.p, hist, wtot);
    wg_signal<false>(&a.ctl[kCtlReady]);
  }
}

// y[t, 128 features of block cb] for the listed tokens: 16 bytes per thread, fp32 accumulation in
// slot order (the arithmetic of the combine kernel).
__device__ __forceinline__ void decode_combine(const DecodeArgs& a, const int* s_list, int nl, int cb) {
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

__global__ void __launch_bounds__(256, 3) decode_layer_kernel(const DecodeArgs a) {
  extern __shared__ __align__(16) unsigned char smem[];
  __shared__ int s_word[2];
  __shared__ int s_list[kDecMaxT];
  __shared__ int s_nlist;
  __shared__ int s_up[kMaxExperts + 1], s_dn[kMaxExperts + 1];   // units before expert e (experts with rows only)
  __shared__ int s_wsum[4][2];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int total = (int)gridDim.x;
  int* const up_done = a.ctl + kDecCtlHead;      // finished up units per expert
  int* const done_list = up_done + a.r.Ne;       // experts in the order in which their up units became complete (e + 1)
  int* const tok_done = done_list + (size_t)a.r.Ne * kDoneStride;      // finished down units per (token, feature block)
  long long* const tr = threadIdx.x == 0 ? a.trace : nullptr;

  // ---- first queue: the router (route tasks, then select tasks) ------------------------------------
  const int nA = a.n_route + a.n_select;
  for (;;) {
    int i = 0;
    if (threadIdx.x == 0) i = draw(&a.ctl[kCtlNextA]);
    i = wg_bcast(i, &s_word[0]);
    if (i < 0 || i >= nA) {
      // (a negative index can only come from counters that were not zero at the start)
      if (i < 0 && threadIdx.x == 0) set_failed(a, 2);
      break;
    }
    if (tr) tr[(size_t)i * 4] = __builtin_amdgcn_s_memrealtime();
    if (i < a.n_route) {
      decode_route_partial(a, i, smem, lane, w);
      wg_signal<true>(&a.ctl[kCtlParts]);
    } else {
      decode_select(a, i - a.n_route, smem, s_word, lane, w);
    }
    if (tr) tr[(size_t)i * 4 + 3] = __builtin_amdgcn_s_memrealtime();
  }

  // ---- everybody: wait for the routing, then the tables of the units that have rows -----------------
  const bool ready = wg_wait(a, &a.ctl[kCtlReady], 1, &s_word[1]);
  int U = 0, D = 0;
  if (ready) {
    // thread e: expert e.  What was published is used as indices only if it is consistent (rows
    // inside [0, P), at most T of them); anything else means the counters were not zero at the
    // start and let this workgroup run ahead of the permutation: the expert is left out.
    const int e = threadIdx.x;
    int nu = 0, nd = 0;
    if (e < a.r.Ne) {
      const int row0 = a.p.offsets[e], cnt = a.p.offsets[e + 1] - row0;
      if (cnt != 0) {
        if (row0 >= 0 && cnt > 0 && cnt <= a.r.T && row0 + cnt <= a.p.P) {
          nu = a.up.F[e / a.r.N] / 64;
          nd = a.ncb;
        } else {
          set_failed(a, 2);
        }
      }
    }
    int iu = nu, id = nd;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int xu = __shfl_up(iu, off, 64), xd = __shfl_up(id, off, 64);
      if (lane >= off) { iu += xu; id += xd; }
    }
    if (lane == 63) { s_wsum[w][0] = iu; s_wsum[w][1] = id; }
    __syncthreads();
    int bu = 0, bd = 0;
    for (int ww = 0; ww < w; ++ww) { bu += s_wsum[ww][0]; bd += s_wsum[ww][1]; }
    if (e < a.r.Ne) {
      s_up[e] = bu + iu - nu;
      s_dn[e] = bd + id - nd;
    }
    if (e == a.r.Ne - 1) {                   // entry Ne: the totals
      s_up[a.r.Ne] = bu + iu;
      s_dn[a.r.Ne] = bd + id;
    }
    __syncthreads();
    U = s_up[a.r.Ne];
    D = s_dn[a.r.Ne];
  }

  // ---- second queue: up units, then down units, of the experts that have rows -------------------------
  int j = 0;
  if (threadIdx.x == 0) j = ready ? draw(&a.ctl[kCtlNextB]) : U + D;
  j = wg_bcast(j, &s_word[0]);
  while (j >= 0 && j < U + D) {
    // the next draw is requested now and used after this unit.  (A drawn unit that has not been
    // started is always later in the queue than the one in hand, so nothing a waiting down unit
    // depends on can be held back by it: up units never wait.)
    int jn = 0;
    if (threadIdx.x == 0) jn = draw(&a.ctl[kCtlNextB]);
    const bool isup = j < U;
    const int jj = isup ? j : j - U;
    long long* const tu = tr ? tr + ((size_t)nA + j) * 4 : nullptr;
    if (tu) tu[0] = __builtin_amdgcn_s_memrealtime();
    int e = 0, cb = 0;
    bool have = true;
    if (isup) {
      // up units: expert by expert in index order
      if ((int)threadIdx.x < a.r.Ne && s_up[threadIdx.x] <= jj && jj < s_up[threadIdx.x + 1]) s_word[1] = threadIdx.x;
      __syncthreads();
      e = s_word[1];
      cb = jj - s_up[e];
    } else {
      // down units: the experts in the order in which their up units became complete, so that a
      // unit waits only when no expert at all is ready for it
      const int q = jj / a.ncb;
      cb = jj - q * a.ncb;
      const int v = wg_wait_value(a, &done_list[(q < a.r.Ne ? q : a.r.Ne - 1) * kDoneStride], &s_word[1]);
      e = v - 1;
      have = v > 0 && e < a.r.Ne && s_dn[e + 1] > s_dn[e];
      if (!have) e = 0;
      if (tu) tu[1] = __builtin_amdgcn_s_memrealtime();
    }
    const int g = e / a.r.N;
    const int row0 = a.p.offsets[e], cnt = have ? a.p.offsets[e + 1] - row0 : 0;
    // the pairs named by the expert's rows must lie in [0, P) before they are used as indices
    __syncthreads();
    if (threadIdx.x == 0) s_nlist = 0;
    __syncthreads();
    if ((int)threadIdx.x < cnt) {
      const int pr = a.p.perm[row0 + threadIdx.x];
      if (pr < 0 || pr >= a.p.P) s_nlist = -1;
    }
    __syncthreads();
    const bool rows_ok = s_nlist == 0;
    __syncthreads();
    if (!have) {
      // (the wait expired, or the list named no expert with rows: the failure word says which)
      if (threadIdx.x == 0) set_failed(a, 1);
    } else if (!rows_ok) {
      if (threadIdx.x == 0) set_failed(a, 2);
    } else if (isup) {
      skinny_unit<true, true>(a.up, a.up.blk_prefix[g] + (e - g * a.r.N) * (a.up.F[g] / 64) + cb);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this wave's rows of H are written through
      __syncthreads();
      if (threadIdx.x == 0) {
        // the unit that completes the expert appends it to the list the down units are taken from
        const int old = __hip_atomic_fetch_add(&up_done[e], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old == a.up.F[g] / 64 - 1) {
          const int at = __hip_atomic_fetch_add(&a.ctl[kCtlDoneTail], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (at >= 0 && at < a.r.Ne) __hip_atomic_store(&done_list[at * kDoneStride], e + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    } else {
      skinny_unit<false, true>(a.dn, a.dn.blk_prefix[g] + (e - g * a.r.N) * a.ncb + cb);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // this wave's rows of y_perm are written through
      __syncthreads();
      // one thread per routed row of the expert: its token's counter for this feature block
      for (int tt = threadIdx.x; tt < cnt; tt += blockDim.x) {
        const int t = a.p.perm[row0 + tt] / a.dn.Ke;
        const int old = __hip_atomic_fetch_add(&tok_done[t * a.ncb + cb], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old == a.dn.Ke - 1) {
          // (the other K_e - 1 units of this token finished before: their rows, written through and
          // never read by this XCD so far, are read next)
          const int at = atomicAdd(&s_nlist, 1);
          if (at < kDecMaxT) s_list[at] = t;
        }
      }
      __syncthreads();
      decode_combine(a, s_list, s_nlist < kDecMaxT ? s_nlist : kDecMaxT, cb);
    }
    if (tu) tu[3] = __builtin_amdgcn_s_memrealtime();
    j = wg_bcast(jn, &s_word[0]);
  }
  if (j < 0 && threadIdx.x == 0) set_failed(a, 2);

  // ---- the last workgroup to leave clears the control words for the next call -------------------
  __syncthreads();
  if (threadIdx.x == 0) {
    // (this thread issued the workgroup's counter updates: they have been performed before it leaves)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    s_word[1] = __hip_atomic_fetch_add(&a.ctl[kCtlExited], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  if (s_word[1] == total - 1) {
    const int failed = ctl_load(&a.ctl[kCtlFailed]);
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(a.status, failed, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (int i = threadIdx.x; i < a.n_ctl; i += blockDim.x) a.ctl[i] = 0;
    if (failed) poison_y(a);
  } else if (s_word[1] < 0 || s_word[1] >= total) {
    // no workgroup will find itself the last: the counters were not zero at the start
    if (threadIdx.x == 0) __hip_atomic_store(a.status, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (blockIdx.x == 0) poison_y(a);
  }
}

// ---- host ------------------------------------------------------------------------------------------
struct DecodeLayout {
  size_t ctl, status, gpart, counts, offsets, perm, inv_perm, h, y_perm, total;
  int n_ctl, ncb, NS, NSP;
};

static DecodeLayout decode_layout(const LayerDesc& L) {
  DecodeLayout o;
  auto up256 = [](size_t b) { return (b + 255) / 256 * 256; };
  o.ncb = (L.d + 127) / 128;
  o.NS = (L.d + 4 * kDecSlice - 1) / (4 * kDecSlice);     // partial sums per logit ...
  o.NSP = (o.NS + 1) / 2 * 2;                              // ... stored with an even pitch (read in pairs)
  o.n_ctl = kDecCtlHead + L.Ne + L.Ne * kDoneStride + L.T * o.ncb;
  size_t at = 0;
  o.ctl = at; at += up256((size_t)o.n_ctl * sizeof(int));
  o.status = at; at += 256;
  o.gpart = at; at += up256((size_t)o.NSP * L.T * (L.Ng + L.Ne) * sizeof(double));   // [T][N_g + N_e][NS]
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
                               float* gates, void* y, void* ws, int spin_limit, long long* trace, hipStream_t s) {
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
  a.NSP = lay.NSP;
  a.n_route = a.TB * a.OT * a.NS;
  a.n_select = (L.T + kDecSelTokens - 1) / kDecSelTokens;
  a.n_up = nu;
  a.n_down = nd;
  a.ncb = lay.ncb;
  a.gates = gates;
  a.y = static_cast<uint16_t*>(y);
  a.spin_limit = spin_limit == 0 ? kDecSpinLimit : spin_limit;
  a.trace = trace;
  const size_t sel = (size_t)r.region0 + (size_t)kDecSelTokens * r.NOpad * sizeof(float);
  const size_t srt = sizeof(int) * (kWavesPerBlock * kMaxExperts + kWavesPerBlock);
  const size_t red = (size_t)4 * 256 * sizeof(double);        // the route task's reduction over its waves
  const size_t smem = sel > srt ? (sel > red ? sel : red) : (srt > red ? srt : red);
  // persistent workgroups: as many as the device holds at once, no more than there are pieces of work
  // (progress does not depend on their all being resident: work is drawn in dependency order)
  static size_t occ_smem = ~(size_t)0;
  static int occ_blocks = 0;
  if (occ_smem != smem) {
    int nb = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, decode_layer_kernel, 256, smem) != hipSuccess || nb < 1) nb = 1;
    occ_blocks = nb;
    occ_smem = smem;
  }
  int dev = 0, cus = 256;
  hipDeviceProp_t prop;
  static int cached_cus = 0;
  if (!cached_cus) {
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount > 0)
      cus = prop.multiProcessorCount;
    cached_cus = cus;
  }
  long long grid = (long long)cached_cus * occ_blocks;
  const long long work = (long long)a.n_route + a.n_select + a.n_up + a.n_down;
  if (grid > work) grid = work;
  if (grid < 1) grid = 1;
  hipLaunchKernelGGL(decode_layer_kernel, dim3((unsigned)grid), dim3(256), smem, s, a);
  return hipGetLastError();
}

// pieces of work of a call at most (route tasks, select tasks, all units): entries of the optional trace
long long decode_layer_trace_entries(const LayerDesc& L) {
  const DecodeLayout lay = decode_layout(L);
  long long n = (long long)((L.T + 15) / 16) * ((L.Ng + L.Ne + 15) / 16) * lay.NS + (L.T + kDecSelTokens - 1) / kDecSelTokens;
  for (int g = 0; g < L.Ng; ++g) n += (long long)L.N * (L.F[g] / 64 + lay.ncb);
  return n;
}

long long decode_layer_status_offset(const LayerDesc& L) { return (long long)decode_layout(L).status; }

}  // namespace mohge
