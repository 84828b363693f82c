// Expert feed-forward networks for decode-sized token counts on gfx950 (a handful of
// tokens per expert): bandwidth-bound, every touched expert's weights are streamed once.
//
// A wave owns 2 x 16 weight rows (up: 16 W_gate rows and the matching 16 W_up rows;
// down: 32 consecutive W_down rows) and runs over the whole reduction dimension with
// v_mfma_f32_16x16x32_bf16, the weight rows as the first operand and up to 32 of the
// expert's tokens as the second.  Lanes load 16 contiguous bytes of "their" weight row,
// which is the operand layout, so weights go global -> registers -> matrix core with no
// LDS traffic; token rows come through L1/L2 (lanes past the token count load nothing).
// Experts without tokens are skipped on the device: their workgroups exit at once.
//
// Quantised weights (ffn_skinny_q_kernel): FP8 E4M3 codes with one fp32 scale per weight row, or
// MXFP4 (E2M1 codes, two to a byte, an E8M0 scale per block of 32 elements of the reduction
// dimension).  A lane still loads 16 contiguous bytes of its weight row: 16 FP8 codes, which the
// hardware conversion turns into two bf16 operand fragments (E4M3 values are exact in bf16; the
// row scale multiplies the fp32 sum in the epilogue), or one MXFP4 block, which the hardware
// conversion (E2M1 pair x power-of-two scale -> packed bf16, exact) turns into four, so that the
// scaling happens before the matrix core.  The token operand is read with the same assignment of
// reduction indices to operand slots.
#include <type_traits>

#include "common.h"
#include "skinny.h"

namespace mohge {

template <bool UP>
__global__ void __launch_bounds__(256) ffn_skinny_kernel(const SkinnyArgs a) {
  skinny_unit<UP, false>(a, (int)blockIdx.x);
}

// 16 E4M3 codes -> two operand fragments of 8 bf16 (codes 0..7 and 8..15)
__device__ __forceinline__ void fp8x16_to_bf16(const uint4 c, Frag& lo, Frag& hi) {
  const uint32_t w[4] = {c.x, c.y, c.z, c.w};
  uint32_t o[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 a = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], false);   // codes 0, 1 of the word
    const f32x2 b = __builtin_amdgcn_cvt_pk_f32_fp8((int)w[i], true);    // codes 2, 3
    // exact in bf16: keep the upper halves of the fp32 patterns
    o[2 * i] = (__float_as_uint(a[0]) >> 16) | (__float_as_uint(a[1]) & 0xffff0000u);
    o[2 * i + 1] = (__float_as_uint(b[0]) >> 16) | (__float_as_uint(b[1]) & 0xffff0000u);
  }
  lo.u = make_uint4(o[0], o[1], o[2], o[3]);
  hi.u = make_uint4(o[4], o[5], o[6], o[7]);
}

// E8M0 code -> the power of two as fp32 bits (code 0: 2^-127, a subnormal; 255: NaN)
__device__ __forceinline__ float e8m0_to_f32(uint32_t c) {
  const uint32_t bits = c == 0u ? 0x00400000u : (c == 255u ? 0x7fc00000u : c << 23);
  return __uint_as_float(bits);
}

// 8 E2M1 codes (one word, element 2j in the low half of byte j) times the block scale -> 8 bf16
__device__ __forceinline__ void fp4x8_to_bf16(const uint32_t c, const float scale, Frag& o) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  union { bf16x2 v; uint32_t u; } p0, p1, p2, p3;
  p0.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(c, scale, 0);
  p1.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(c, scale, 1);
  p2.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(c, scale, 2);
  p3.v = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(c, scale, 3);
  o.u = make_uint4(p0.u, p1.u, p2.u, p3.u);
}

// Quantised-weight variant of ffn_skinny_kernel (BITS = 8: FP8 E4M3, BITS = 4: MXFP4): same split
// of the weight rows over workgroups and waves.  A unit of the reduction is 64 bytes of a weight
// row: lane (r, q) holds 16 bytes of its row, 16 (FP8) or 32 (MXFP4) consecutive indices, used as
// two or four MFMA steps.  With fewer bytes per weight, keeping the memory system busy takes more
// loads in flight per wave than token fragments held in registers leave room for, so here
//  - the expert's tokens (16 per pass) are staged once per workgroup in LDS, in chunks of the
//    reduction dimension sized to the token count (all of it for a handful of tokens), and read
//    from there right before each MFMA; rows are padded by 16 bytes against bank conflicts and
//    zero-filled past the reduction length, so that cut-short units need no special case;
//  - MXFP4: the block scales of the workgroup's 128 weight rows are staged in LDS with the tokens
//    (a scale byte per lane and block straight from memory is a 16-line request for 64 bytes,
//    and those lines do not survive in the vector cache between steps);
//  - the weights of the next step (4 units) are requested before the current one is converted
//    and multiplied.
// Token columns past the expert's count hold copies of its last staged token; MFMA columns are
// independent and those outputs are never stored.
constexpr int kStageBytes = 22528;            // token rows; with the scales 40 KB: four workgroups per CU
constexpr int kScaleChunk = 4096;             // longest chunk of the reduction dimension
constexpr int kScalePitch = kScaleChunk / 32 + 16;   // 16-byte aligned rows, 36 dwords apart: no bank conflicts
constexpr int kScaleBytes = 128 * kScalePitch;

template <bool UP, int BITS>
__global__ void __launch_bounds__(256) ffn_skinny_q_kernel(const SkinnyArgs a) {
  static_assert(BITS == 4 || BITS == 8, "MXFP4 or FP8 codes");
  constexpr int UK = 512 / BITS;              // reduction indices per unit: 64 bytes of a weight row
  constexpr int LK = UK / 4;                  // ... per lane
  constexpr int NJ = LK / 8;                  // MFMA steps per unit
  __shared__ uint4 xs[kStageBytes / 16];
  __shared__ uint32_t ss[BITS == 4 ? kScaleBytes / 4 : 4];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int r = lane & 15, q = lane >> 4;
  int g = 0;
  while (g + 1 < a.Ng && (int)blockIdx.x >= a.blk_prefix[g + 1]) ++g;
  const int F = a.F[g];
  const int K = UP ? a.d : F;
  const int ncols = UP ? F : a.d;
  constexpr int COLS_PER_BLOCK = UP ? 64 : 128;
  const int blocks_per_expert = (ncols + COLS_PER_BLOCK - 1) / COLS_PER_BLOCK;
  const int local = blockIdx.x - a.blk_prefix[g];
  const int i = local / blocks_per_expert, cb = local % blocks_per_expert;
  const int e = g * a.N + i;
  const int row0 = a.offsets[e], cnt = a.offsets[e + 1] - row0;
  if (cnt <= 0) return;                       // the whole workgroup
  const int c0 = cb * COLS_PER_BLOCK + w * (UP ? 16 : 32);
  const bool active = c0 < ncols;             // idle waves still stage tokens and meet the barriers

  long long wrow[2] = {0, 0};
  if (active) {
    if constexpr (UP) {
      wrow[0] = (long long)i * 2 * F + c0 + r;
      wrow[1] = (long long)i * 2 * F + F + c0 + r;
    } else {
      int n1 = c0 + 16 + r;
      if (n1 > a.d - 1) n1 = a.d - 1;
      wrow[0] = (long long)i * a.d + c0 + r;
      wrow[1] = (long long)i * a.d + n1;
    }
  }
  const uint8_t* wbase = reinterpret_cast<const uint8_t*>(a.W[g]);
  const uint8_t* wp[2] = {wbase + wrow[0] * (K * BITS / 8) + 16 * q, wbase + wrow[1] * (K * BITS / 8) + 16 * q};
  // rows of the staged scales: this lane's two weight rows
  const uint8_t* const slds = reinterpret_cast<const uint8_t*>(ss);
  const uint8_t* sp[2];
  if constexpr (UP) {
    sp[0] = slds + (16 * w + r) * kScalePitch + q;
    sp[1] = slds + (64 + 16 * w + r) * kScalePitch + q;
  } else {
    sp[0] = slds + (32 * w + r) * kScalePitch + q;
    sp[1] = slds + (32 * w + 16 + r) * kScalePitch + q;
  }

  constexpr int U = 4;                        // units per step
  const int Kp = (K + 127) & ~127;            // staged length: zero-filled past K
  unsigned char* const lds = reinterpret_cast<unsigned char*>(xs);

  for (int tb0 = 0; tb0 < cnt; tb0 += 16) {
    const int ns = min(cnt - tb0, 16);        // tokens of this pass
    // chunk of the reduction dimension whose ns rows fit the staging buffer
    int KC = Kp < kScaleChunk ? Kp : kScaleChunk;
    while (ns * (KC * 2 + 16) > kStageBytes) KC = ((KC >> 1) + 127) & ~127;
    const int pitch = KC * 2 + 16;
    const unsigned char* xrow = lds + (r < ns ? r : ns - 1) * pitch + 2 * LK * q;

    f32x4 acc[2];
    acc[0] = f32x4{0.f, 0.f, 0.f, 0.f};
    acc[1] = f32x4{0.f, 0.f, 0.f, 0.f};

    // weights of the step at k0 inside the chunk that ends at cend
    auto load = [&](uint4 (&wq)[2][U], int k0, int cend) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int k = k0 + UK * u;
        const bool kv = k < cend && k + LK * q < K;
#pragma unroll
        for (int f = 0; f < 2; ++f) {
          wq[f][u] = make_uint4(0u, 0u, 0u, 0u);
          if (kv) wq[f][u] = *reinterpret_cast<const uint4*>(wp[f] + k * BITS / 8);
        }
      }
    };

    // Order of the steps inside a chunk: every wave starts at a different step and wraps around.
    // All weight rows begin at multiples of the row size, a power of two at the usual hidden
    // sizes, so waves that walk in step ask the same few memory channels at any one time;
    // staggered they spread over all of them (a pure-read kernel with this access pattern and
    // 4 KB rows: 5.4-5.8 TB/s in step, 6.3 TB/s staggered; here it is worth 2 %).  The order of the
    // fp32 additions then depends on the wave, which the launch fixes: results stay bit-identical
    // from run to run.
    constexpr int SK = UK * U;                 // indices per step
    const unsigned wave5 = ((unsigned)blockIdx.x * 4u + (unsigned)w) * 5u;
    auto steps_in = [&](int kcx) { return (min(KC, Kp - kcx) + SK - 1) / SK; };
    auto first_pos = [&](int kcx) { return (int)(wave5 % (unsigned)steps_in(kcx)); };

    uint4 wq[2][U];
    int pos = first_pos(0);
    int k0 = pos * SK, cend = min(KC, Kp);
    if (active) load(wq, k0, cend);

    for (int kc = 0; kc < Kp; kc += KC) {
      const int klen = min(KC, Kp - kc);
      // Staging: every global load is issued before the first LDS store, so that a chunk costs
      // about one memory latency; the barrier that protects the previous chunk's readers sits
      // between the loads and the stores.
      const int ppr = klen >> 3;              // 16-byte pieces per token row
      const int npieces = ns * ppr;           // <= kStageBytes / 16 <= 6 * 256 by the choice of KC
      uint4 tv[6];
#pragma unroll
      for (int it = 0; it < 6; ++it) {
        const int idx = threadIdx.x + 256 * it;
        tv[it] = make_uint4(0u, 0u, 0u, 0u);
        if (idx < npieces) {
          const int rr = idx / ppr, c = idx - rr * ppr;
          if (kc + 8 * c < K) {
            const int pos = row0 + tb0 + rr;
            long long src;
            if constexpr (UP) src = a.perm ? (long long)(a.perm[pos] / a.Ke) : (long long)pos;
            else src = pos;
            tv[it] = *reinterpret_cast<const uint4*>(a.A + src * a.lda + kc + 8 * c);
          }
        }
      }
      // MXFP4: block scales of the chunk for the 128 weight rows of the workgroup (code 127 = 1 past K)
      const int nb = BITS == 4 ? klen >> 5 : 0;                                  // blocks per row in the chunk
      const int nbv = ((K < kc + klen ? K : kc + klen) - kc) >> 5;   // of which exist
      const int spitch = K >> 5;
      uint8_t* const sdst = reinterpret_cast<uint8_t*>(ss);
      auto grow = [&](int lr) -> long long {
        if constexpr (UP) return (long long)i * 2 * F + (long long)(lr >> 6) * F + cb * 64 + (lr & 63);
        else {
          int n = cb * 128 + lr;
          if (n > a.d - 1) n = a.d - 1;
          return (long long)i * a.d + n;
        }
      };
      const uint8_t* const sbase = a.S4[g] + (kc >> 5);
      // widest aligned access the shape allows: 16 bytes, 4 bytes, else bytes
      const int sw = BITS != 4 ? 0 : nb != nbv ? 1
                     : (!(spitch & 15) && !((kc >> 5) & 15) && !(nb & 15)) ? 16
                     : (!(spitch & 3) && !((kc >> 5) & 3) && !(nb & 3)) ? 4 : 1;
      uint32_t sv[16];                        // 4 x 16 bytes or 16 x 4 bytes per thread
      if (sw == 16) {
        const int nq = nb >> 4;                                  // <= 8: at most 4 pieces per thread
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int idx = threadIdx.x + 256 * it;
          uint4 v = make_uint4(0u, 0u, 0u, 0u);
          if (idx < 128 * nq) {
            const int lr = idx / nq, c = idx - lr * nq;
            v = *reinterpret_cast<const uint4*>(sbase + grow(lr) * spitch + 16 * c);
          }
          sv[4 * it] = v.x; sv[4 * it + 1] = v.y; sv[4 * it + 2] = v.z; sv[4 * it + 3] = v.w;
        }
      } else if (sw == 4) {
        const int nw = nb >> 2;                                  // <= 32: at most 16 pieces per thread
#pragma unroll
        for (int it = 0; it < 16; ++it) {
          const int idx = threadIdx.x + 256 * it;
          sv[it] = 0u;
          if (idx < 128 * nw) {
            const int lr = idx / nw, c = idx - lr * nw;
            sv[it] = *reinterpret_cast<const uint32_t*>(sbase + grow(lr) * spitch + 4 * c);
          }
        }
      }
      __syncthreads();                        // the previous chunk (or pass) has been consumed
#pragma unroll
      for (int it = 0; it < 6; ++it) {
        const int idx = threadIdx.x + 256 * it;
        if (idx < npieces) {
          const int rr = idx / ppr, c = idx - rr * ppr;
          *reinterpret_cast<uint4*>(lds + rr * pitch + 16 * c) = tv[it];
        }
      }
      if (sw == 16) {
        const int nq = nb >> 4;
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int idx = threadIdx.x + 256 * it;
          if (idx < 128 * nq) {
            const int lr = idx / nq, c = idx - lr * nq;
            *reinterpret_cast<uint4*>(sdst + lr * kScalePitch + 16 * c) =
                make_uint4(sv[4 * it], sv[4 * it + 1], sv[4 * it + 2], sv[4 * it + 3]);
          }
        }
      } else if (sw == 4) {
        const int nw = nb >> 2;
#pragma unroll
        for (int it = 0; it < 16; ++it) {
          const int idx = threadIdx.x + 256 * it;
          if (idx < 128 * nw) {
            const int lr = idx / nw, c = idx - lr * nw;
            *reinterpret_cast<uint32_t*>(sdst + lr * kScalePitch + 4 * c) = sv[it];
          }
        }
      } else if (sw == 1) {
        for (int idx = threadIdx.x; idx < 128 * nb; idx += 256) {
          const int lr = idx / nb, c = idx - lr * nb;
          sdst[lr * kScalePitch + c] = c < nbv ? sbase[grow(lr) * spitch + c] : (uint8_t)127;
        }
      }
      __syncthreads();
      if (!active) continue;
      const int chunk_end = kc + klen;        // == cend of the steps of this chunk
      const int nsteps = steps_in(kc);
      for (int sidx = 0; sidx < nsteps; ++sidx) {
        // request the next step (the first of the next chunk after the last of this one)
        const bool last = sidx + 1 == nsteps;
        int npos = pos + 1 == nsteps ? 0 : pos + 1, nk, ncend;
        if (!last) { nk = kc + npos * SK; ncend = chunk_end; }
        else if (chunk_end < Kp) { npos = first_pos(chunk_end); nk = chunk_end + npos * SK; ncend = min(chunk_end + KC, Kp); }
        else { nk = Kp; ncend = Kp; }
        uint4 wn[2][U];
        load(wn, nk, ncend);                  // loads nothing once nk == Kp
#pragma unroll
        for (int u = 0; u < U; ++u) {
          if (k0 + UK * u < chunk_end) {      // wave-uniform
            const unsigned char* xu = xrow + (k0 - kc + UK * u) * 2;
            Frag xf[NJ];
#pragma unroll
            for (int j = 0; j < NJ; ++j) xf[j].u = *reinterpret_cast<const uint4*>(xu + 16 * j);
#pragma unroll
            for (int f = 0; f < 2; ++f) {
              if constexpr (BITS == 4) {
                const float scale = e8m0_to_f32(sp[f][(k0 - kc + UK * u) >> 5]);
                const uint32_t cw[4] = {wq[f][u].x, wq[f][u].y, wq[f][u].z, wq[f][u].w};
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                  Frag wf;
                  fp4x8_to_bf16(cw[j], scale, wf);
                  acc[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf.v, xf[j].v, acc[f], 0, 0, 0);
                }
              } else {
                Frag wlo, whi;
                fp8x16_to_bf16(wq[f][u], wlo, whi);
                acc[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wlo.v, xf[0].v, acc[f], 0, 0, 0);
                acc[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(whi.v, xf[1].v, acc[f], 0, 0, 0);
              }
            }
          }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int f = 0; f < 2; ++f) wq[f][u] = wn[f][u];
        k0 = nk;
        cend = ncend;
        pos = npos;
      }
    }

    // lane holds token r of the pass, weight rows 4q..4q+3 of each row set
    const int tt = tb0 + r;
    if constexpr (BITS == 8) {
      if (active) {
        // FP8: the scale of the weight row of accumulator element b multiplies the sum
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            long long row;
            if constexpr (UP) row = (long long)i * 2 * F + (long long)f * F + c0 + 4 * q + b;
            else {
              int n = c0 + 16 * f + 4 * q + b;
              if (n > a.d - 1) n = a.d - 1;
              row = (long long)i * a.d + n;
            }
            acc[f][b] *= a.S[g][row];
          }
      }
    }
    if (active && tt < cnt) {
      uint16_t* crow = a.C + (long long)(row0 + tt) * a.ldc;
      if constexpr (UP) {
        float v[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const float gt = acc[0][b], up = acc[1][b];
          v[b] = gt / (1.f + __expf(-gt)) * up;
        }
        uint2 o;
        o.x = pack_bf16x2(v[0], v[1]);
        o.y = pack_bf16x2(v[2], v[3]);
        *reinterpret_cast<uint2*>(crow + c0 + 4 * q) = o;
      } else {
#pragma unroll
        for (int f = 0; f < 2; ++f) {
          const int col = c0 + 16 * f + 4 * q;
          if (col < ncols) {
            uint2 o;
            o.x = pack_bf16x2(acc[f][0], acc[f][1]);
            o.y = pack_bf16x2(acc[f][2], acc[f][3]);
            *reinterpret_cast<uint2*>(crow + col) = o;
          }
        }
      }
    }
  }
}

// MXFP4 -> fp32 through the conversion the kernel uses (a thread per block of 32), for checks and tools
__global__ void __launch_bounds__(256) mxfp4_decode_kernel(const uint32_t* __restrict__ packed,
                                                           const uint8_t* __restrict__ scales,
                                                           float* __restrict__ out, long long nblocks) {
  const long long b = (long long)blockIdx.x * 256 + threadIdx.x;
  if (b >= nblocks) return;
  const float scale = e8m0_to_f32(scales[b]);
  for (int j = 0; j < 4; ++j) {
    Frag f;
    fp4x8_to_bf16(packed[4 * b + j], scale, f);
    const uint32_t wv[4] = {f.u.x, f.u.y, f.u.z, f.u.w};
    for (int t = 0; t < 4; ++t) {
      out[32 * b + 8 * j + 2 * t] = __uint_as_float(wv[t] << 16);
      out[32 * b + 8 * j + 2 * t + 1] = __uint_as_float(wv[t] & 0xffff0000u);
    }
  }
}

hipError_t launch_mxfp4_decode(const void* packed, const void* scales, float* out, long long n, hipStream_t s) {
  const long long nb = n / 32;
  if (nb <= 0) return hipSuccess;
  hipLaunchKernelGGL(mxfp4_decode_kernel, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, s,
                     static_cast<const uint32_t*>(packed), static_cast<const uint8_t*>(scales), out, nb);
  return hipGetLastError();
}

// codes -> fp32, for checks and tools
__global__ void __launch_bounds__(256) fp8_decode_kernel(const uint8_t* __restrict__ q, float* __restrict__ out,
                                                         long long n) {
  const long long i = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;
  if (i >= n) return;
  uint32_t wv = 0;
  for (int b = 0; b < 4; ++b)
    if (i + b < n) wv |= (uint32_t)q[i + b] << (8 * b);
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)wv, false), hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)wv, true);
  const float v[4] = {lo[0], lo[1], hi[0], hi[1]};
  for (int b = 0; b < 4; ++b)
    if (i + b < n) out[i + b] = v[b];
}

hipError_t launch_fp8_decode(const void* q, float* out, long long n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(fp8_decode_kernel, dim3((unsigned)((n + 1023) / 1024)), dim3(256), 0, s,
                     static_cast<const uint8_t*>(q), out, n);
  return hipGetLastError();
}

// Argument blocks of the up and the down launch (one workgroup per unit: nu / nd of them)
void skinny_args(const LayerDesc& L, const void* x, const int32_t* perm, const int32_t* offsets,
                 const GroupPtrs& W, void* y_perm, void* h, const float* const* s13, const float* const* s2,
                 const void* const* b13, const void* const* b2, SkinnyArgs& up, SkinnyArgs& dn, int& nu, int& nd) {
  const bool w8 = s13 != nullptr, w4 = b13 != nullptr;
  up.A = static_cast<const uint16_t*>(x);
  up.perm = perm;
  up.offsets = offsets;
  up.C = static_cast<uint16_t*>(h);
  up.lda = L.d; up.ldc = L.Fmax; up.Ke = L.Ke; up.Ng = L.Ng; up.N = L.N; up.d = L.d;
  dn = up;
  dn.A = static_cast<const uint16_t*>(h);
  dn.perm = nullptr;
  dn.C = static_cast<uint16_t*>(y_perm);
  dn.lda = L.Fmax; dn.ldc = L.d;
  nu = 0; nd = 0;
  for (int g = 0; g < kMaxGroups; ++g) {
    up.F[g] = dn.F[g] = g < L.Ng ? L.F[g] : 0;
    up.W[g] = static_cast<const uint16_t*>(W.w13[g]);
    dn.W[g] = static_cast<const uint16_t*>(W.w2[g]);
    up.S[g] = w8 && g < L.Ng ? s13[g] : nullptr;
    dn.S[g] = w8 && g < L.Ng ? s2[g] : nullptr;
    up.S4[g] = w4 && g < L.Ng ? static_cast<const uint8_t*>(b13[g]) : nullptr;
    dn.S4[g] = w4 && g < L.Ng ? static_cast<const uint8_t*>(b2[g]) : nullptr;
    up.blk_prefix[g] = nu;
    dn.blk_prefix[g] = nd;
    if (g < L.Ng) {
      nu += L.N * (L.F[g] / 64);
      nd += L.N * ((L.d + 127) / 128);
    }
  }
  up.blk_prefix[kMaxGroups] = nu;
  dn.blk_prefix[kMaxGroups] = nd;
}

hipError_t launch_ffn_skinny(const LayerDesc& L, const void* x, const int32_t* perm,
                             const int32_t* offsets, const GroupPtrs& W, void* y_perm, void* ws,
                             hipStream_t s, int stages, const float* const* s13, const float* const* s2,
                             const void* const* b13, const void* const* b2) {
  const bool w8 = s13 != nullptr, w4 = b13 != nullptr;
  SkinnyArgs up, dn;
  int nu = 0, nd = 0;
  skinny_args(L, x, perm, offsets, W, y_perm, ws, s13, s2, b13, b2, up, dn, nu, nd);
  if (w4) {
    if (stages & 1) hipLaunchKernelGGL((ffn_skinny_q_kernel<true, 4>), dim3(nu), dim3(256), 0, s, up);
    if (stages & 2) hipLaunchKernelGGL((ffn_skinny_q_kernel<false, 4>), dim3(nd), dim3(256), 0, s, dn);
    return hipGetLastError();
  }
  if (w8) {
    if (stages & 1) hipLaunchKernelGGL((ffn_skinny_q_kernel<true, 8>), dim3(nu), dim3(256), 0, s, up);
    if (stages & 2) hipLaunchKernelGGL((ffn_skinny_q_kernel<false, 8>), dim3(nd), dim3(256), 0, s, dn);
    return hipGetLastError();
  }
  if (stages & 1) hipLaunchKernelGGL((ffn_skinny_kernel<true>), dim3(nu), dim3(256), 0, s, up);
  if (stages & 2) hipLaunchKernelGGL((ffn_skinny_kernel<false>), dim3(nd), dim3(256), 0, s, dn);
  return hipGetLastError();
}

}  // namespace mohge
