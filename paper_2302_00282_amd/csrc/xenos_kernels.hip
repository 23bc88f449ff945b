// gfx950 (CDNA4) kernels of the linked-operator-chain path.
//
//  conv_kernel   implicit-GEMM dense convolution on MFMA (bf16 32x32x16 / fp32 32x32x2, fp32
//                accumulate) with the whole linked chain in its epilogue: folded BN/bias scale+shift,
//                shortcut add, ReLU, max/avg/global pooling, and a store at a channel offset of the
//                consumer's buffer (CBR / CBRM / CBRA of Table 3; shortcut and concat rows of Table 1).
//  dw_kernel     depthwise convolution chain (Section 2.2), channel-vectorised NHWC.
//  elt/pool/cvt  stand-alone passes used by the un-linked baselines and at the graph boundary.
//
// Rows of a GEMM tile are conv-output pixels, columns are output channels, the reduction runs over
// (r, s, c) with c fastest, which is contiguous in NHWC.  Output-channel tiles are the paper's
// outC-first partition, pixel tiles its inH/inW partition (Section 4.2.1); the (c, r, s) loop is the
// in-unit parameter split (Section 4.2.2) and never crosses workgroups.
#include "device_common.h"

namespace xenos {

// ---------------------------------------------------------------------------------------------
// Dense convolution chain
// ---------------------------------------------------------------------------------------------
constexpr int STG_PAD = 4;       // staging row pitch = BN + 4 floats (keeps 16-byte alignment of channel groups)

template <int BM, int BN>
__host__ __device__ constexpr int lds_conv_bytes() { return cmax(2 * (BM + BN) * LDS_ROW, BM * (BN + STG_PAD) * 4); }

// DWPRO: the A operand is not read from memory but produced on the fly by a linked depthwise 3x3 convolution
// (+ scale/shift + ReLU) of the tensor `in`: the depthwise output never exists in HBM (Section 2.2: the depthwise
// producer hands its result to the pointwise consumer in the consumer's channel-first order).
template <typename T, int BM, int BN, int WM, int WN, bool SCALAR, int MODE, bool DWPRO = false>
__global__ __launch_bounds__(NT, 2) void conv_kernel(const ConvArgs a) {
  using tr = Tr<T>;
  constexpr int CE = tr::CE, BKE = tr::BKE;
  constexpr int WAVES_N = BN / WN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int A_CH = BM * CPR, B_CH = BN * CPR;                      // 16-byte chunks per step
  constexpr int A_IT = (A_CH + NT - 1) / NT, B_IT = (B_CH + NT - 1) / NT;
  constexpr int SP = BN + STG_PAD;                                 // staging pitch in floats
  constexpr int CG = BN / CE;                                      // channel groups (16-byte stores) per row
  static_assert((BM / WM) * WAVES_N == 4, "four wavefronts per workgroup");

  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
  const int l31 = lane & 31, lhalf = lane >> 5;

  const int nsteps_all = a.Kred_pad / BKE;
  const int OHW = a.OH * a.OW;
  const int ksplit = a.ksplit >= 1 ? a.ksplit : 1;                 // reduction split across workgroups (C/R/S split)
  const bool partial = a.ksplit >= 1;                              // raw fp32 sums go to `part` (even with a single share)
  // Workgroups are dealt round-robin to the 8 XCDs.  The XCDs form an xm x (8/xm) grid over (pixel tiles) x
  // (channel tiles x reduction shares); each owns a contiguous, balanced block of that space and walks its pixel
  // tiles once per channel tile, so at any time the workgroups of one XCD share one weight slice in their L2 and
  // neighbouring pixel tiles share their input halo.  xm = 8 when there are many pixel tiles; problems with few
  // pixel tiles (batch 1, fully connected layers) spread the channel tiles over the XCDs instead.
  const int xm = a.xcd_m, xn = NUM_XCD / xm;
  const int NZ = a.tiles_n * ksplit;
  const int mchunk = (a.tiles_m + xm - 1) / xm, zchunk = (NZ + xn - 1) / xn;
  const int slots = mchunk * zchunk * NUM_XCD;

  for (int t = blockIdx.x; t < slots; t += gridDim.x) {
    const int xcd = t % NUM_XCD, j = t / NUM_XCD;
    const int xi = xcd % xm, xj = xcd / xm;
    const int m0 = xi * a.tiles_m / xm, m1 = (xi + 1) * a.tiles_m / xm;
    const int z0 = xj * NZ / xn, z1 = (xj + 1) * NZ / xn;
    const int lm = j % mchunk, lz = j / mchunk;
    if (lm >= m1 - m0 || lz >= z1 - z0) continue;                  // uniform per workgroup
    const int tile_m = m0 + lm;
    const int tile_n = (z0 + lz) / ksplit, zsplit = (z0 + lz) % ksplit;
    // this workgroup's share of the reduction steps: [s_begin, s_begin + nsteps)
    const int s_begin = partial ? zsplit * a.steps_per_split : 0;
    const int nsteps = partial ? (nsteps_all - s_begin < a.steps_per_split ? nsteps_all - s_begin : a.steps_per_split) : nsteps_all;

    // patch / gap geometry of this tile
    int img = 0, oy0 = 0, ox0 = 0, py = 0, px = 0;
    if (MODE == M_PATCH) {
      const int pper = a.patches_y * a.patches_x;
      img = tile_m / pper;
      const int pr = tile_m % pper;
      py = pr / a.patches_x; px = pr % a.patches_x;
      oy0 = py * a.pph * a.ps - a.pp;
      ox0 = px * a.ppw * a.ps - a.pp;
    } else if (MODE == M_GAP) {
      img = tile_m;
    }
    const int nchunks = (MODE == M_GAP) ? (OHW + BM - 1) / BM : 1;
    float gsum = 0.f;                                              // M_GAP: this thread's column partial sum

    for (int mc = 0; mc < nchunks; ++mc) {
      // ---- decode the rows this thread loads ---------------------------------------------------
      int ih0[A_IT], iw0[A_IT];
      long long rbase[A_IT];
      const int ch = tid % CPR;
#pragma unroll
      for (int it = 0; it < A_IT; ++it) {
        const int row = (tid + it * NT) / CPR;
        int n = 0, oh = 0, ow = 0;
        bool ok = row < BM;
        if (MODE == M_FLAT) {
          const int m = tile_m * BM + row;
          ok = ok && m < a.M_total;
          n = m / OHW; const int p = m - n * OHW; oh = p / a.OW; ow = p - oh * a.OW;
        } else if (MODE == M_ZIGZAG) {
          const int m = tile_m * BM + row;
          ok = ok && m < a.M_total;
          const int wdx = m >> 2, j = m & 3, pw_ = a.PH * a.PW;
          n = wdx / pw_; const int q = wdx - n * pw_; const int ph = q / a.PW;
          oh = 2 * ph + (j >> 1); ow = 2 * (q - ph * a.PW) + (j & 1);
        } else if (MODE == M_PATCH) {
          const int cy = row / a.patch_w, cx = row - cy * a.patch_w;
          n = img; oh = oy0 + cy; ow = ox0 + cx;
          ok = ok && cy < a.patch_h && oh >= 0 && oh < a.OH && ow >= 0 && ow < a.OW;
        } else {
          const int p = mc * BM + row;
          ok = ok && p < OHW;
          n = img; oh = p / a.OW; ow = p - oh * a.OW;
        }
        ih0[it] = ok ? oh * a.stride - a.pad : -(1 << 28);
        iw0[it] = ow * a.stride - a.pad;
        // element offset of input pixel (ih0, iw0); only ever dereferenced together with an in-range tap
        rbase[it] = ok ? (long long)n * a.in_sN + (long long)ih0[it] * a.in_sH + (long long)iw0[it] * a.in_sW : 0;
        if (DWPRO) rbase[it] = ok ? (long long)n * a.dw_sN : 0;    // image base of the depthwise input; (ih0, iw0) = pointwise pixel
      }
      // reduction position (r, s, c) of this thread's 16-byte chunk
      int kc, kr, ks;
      {
        if (a.kchunk) {
          const int rs_n = a.R * a.S, cc = s_begin / rs_n, rs = s_begin - cc * rs_n;
          kc = cc * BKE + ch * CE; kr = rs / a.S; ks = rs - kr * a.S;
        } else {
          const int kk = s_begin * BKE + ch * CE;
          kc = kk % a.C; const int rs = kk / a.C; ks = rs % a.S; kr = rs / a.S;
        }
      }
      const unsigned char* wrow[B_IT];
#pragma unroll
      for (int it = 0; it < B_IT; ++it) {
        const int row = (tid + it * NT) / CPR;
        wrow[it] = (const unsigned char*)a.w +
                   ((long long)(tile_n * BN + (row < BN ? row : 0)) * a.Kred_pad + ch * CE) * (long long)sizeof(T);
      }

      f32x16_t acc[TM][TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

      // A ring of D register sets: the operands of step i + D are requested when step i is staged, so a global access
      // has D steps to hide behind.  Timestamps inside the kernel showed a step of a 64 x 64 tile taking half the memory
      // latency (0.46 us, against 0.06 us of MFMA work) with two sets, at batch 1 and at batch 32 alike.  The vector
      // loader is branch-free (out-of-range taps load a dummy address and are zeroed when published), so the number of
      // loads in flight is known statically and only the oldest set is waited for.  (The 128 x 128 tile keeps two sets:
      // its accumulators leave no room for more.)
      constexpr int D = (BM * BN >= 128 * 128) ? 2 : 4;
      u32x4_t ra[D][A_IT], rb[D][B_IT];
      unsigned okm_[D];

      auto load_global = [&](int step, u32x4_t* ra, u32x4_t* rb, unsigned& okm) {
        const int bstep = s_begin + (step < nsteps ? step : nsteps - 1);   // steps past the end re-read valid weights
        if constexpr (DWPRO) {
          // linked depthwise producer: this thread's CE channels of its pixels, fp32 accumulate.  All tap loads of
          // a pixel are issued before any is used (out-of-range taps read a dummy address and are masked), so the
          // step pays one memory latency, not one per tap.
          okm = ~0u;
          const int kcc = kc < a.C ? kc : 0;
#pragma unroll
          for (int it = 0; it < A_IT; ++it) {
            float d[CE];
#pragma unroll
            for (int e = 0; e < CE; ++e) d[e] = 0.f;
            const bool rowok = step < nsteps && kc < a.C && ih0[it] >= 0;
            if (a.dw_k == 3) {
              u32x4_t xr[9], wr[9];
              unsigned m = 0;
#pragma unroll
              for (int t9 = 0; t9 < 9; ++t9) {
                const int ih = ih0[it] * a.dw_stride - a.dw_pad + t9 / 3, iw = iw0[it] * a.dw_stride - a.dw_pad + t9 % 3;
                const bool ok = rowok && (unsigned)ih < (unsigned)a.dw_H && (unsigned)iw < (unsigned)a.dw_W;
                const long long off = ok ? rbase[it] + ((long long)ih * a.dw_W + iw) * a.dw_sP + kcc : kcc;
                xr[t9] = *(const u32x4_t*)((const T*)a.in + off);
                wr[t9] = *(const u32x4_t*)((const T*)a.dw_w + (long long)t9 * a.C + kcc);
                m |= (ok ? 1u : 0u) << t9;
              }
#pragma unroll
              for (int t9 = 0; t9 < 9; ++t9) {
                float x[CE], w[CE];
                tr::unpack(xr[t9], x);
                tr::unpack(wr[t9], w);
                const float keep = ((m >> t9) & 1u) ? 1.f : 0.f;
#pragma unroll
                for (int e = 0; e < CE; ++e) d[e] = fmaf(x[e] * keep, w[e], d[e]);
              }
            } else if (rowok) {
              for (int r = 0; r < a.dw_k; ++r) {
                const int ih = ih0[it] * a.dw_stride - a.dw_pad + r;
                if ((unsigned)ih >= (unsigned)a.dw_H) continue;
                for (int s2 = 0; s2 < a.dw_k; ++s2) {
                  const int iw = iw0[it] * a.dw_stride - a.dw_pad + s2;
                  if ((unsigned)iw >= (unsigned)a.dw_W) continue;
                  float x[CE], w[CE];
                  tr::unpack(*(const u32x4_t*)((const T*)a.in + rbase[it] + ((long long)ih * a.dw_W + iw) * a.dw_sP + kc), x);
                  tr::unpack(*(const u32x4_t*)((const T*)a.dw_w + (long long)(r * a.dw_k + s2) * a.C + kc), w);
#pragma unroll
                  for (int e = 0; e < CE; ++e) d[e] = fmaf(x[e], w[e], d[e]);
                }
              }
            }
            if (rowok) {
#pragma unroll
              for (int e = 0; e < CE; ++e) {
                const float v = d[e] * a.dw_scale[kc + e] + a.dw_shift[kc + e];
                d[e] = a.dw_relu ? fmx(v, 0.f) : v;
              }
            } else {
#pragma unroll
              for (int e = 0; e < CE; ++e) d[e] = 0.f;
            }
            ra[it] = tr::pack(d);
          }
          kc += BKE;
        } else if constexpr (!SCALAR) {
          const bool kok = step < nsteps && kr < a.R && kc < a.C; // false for every step past the end of this share
          const long long koff = (long long)kr * a.in_sH + (long long)ks * a.in_sW + kc;
          okm = 0;
#pragma unroll
          for (int it = 0; it < A_IT; ++it) {
            const int ih = ih0[it] + kr, iw = iw0[it] + ks;
            const bool ok = kok && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
            const long long off = ok ? rbase[it] + koff : 0;
            ra[it] = *(const u32x4_t*)((const T*)a.in + off);
            okm |= (ok ? 1u : 0u) << it;
          }
          if (a.kchunk) {   // channel-chunk major: all taps of one chunk in consecutive steps (halo reuse in cache)
            if (++ks == a.S) { ks = 0; if (++kr == a.R) { kr = 0; kc += BKE; } }
          } else {          // tap major: (r, s) outer, channels inner
            kc += BKE;
            while (kc >= a.C) { kc -= a.C; if (++ks == a.S) { ks = 0; ++kr; } }
          }
        } else {
          okm = ~0u;
          float f[A_IT][CE];
#pragma unroll
          for (int e = 0; e < CE; ++e) {
            const int kk = bstep * BKE + ch * CE + e;
            const int off = a.ktab[2 * kk], rs = a.ktab[2 * kk + 1];
            const int r = rs >> 16, s = rs & 0xffff;
#pragma unroll
            for (int it = 0; it < A_IT; ++it) {
              const int ih = ih0[it] + r, iw = iw0[it] + s;
              const bool ok = step < nsteps && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
              float v = 0.f;
              if (ok) v = a.in_f32 ? ((const float*)a.in)[rbase[it] + off] : tr::ld(a.in, rbase[it] + off);
              f[it][e] = v;
            }
          }
#pragma unroll
          for (int it = 0; it < A_IT; ++it) ra[it] = tr::pack(f[it]);
        }
#pragma unroll
        for (int it = 0; it < B_IT; ++it) rb[it] = *(const u32x4_t*)(wrow[it] + (long long)bstep * ROWB);
      };
      auto store_lds = [&](int stage, const u32x4_t* ra, const u32x4_t* rb, unsigned okm) {
        unsigned char* sa = smem + stage * (BM + BN) * LDS_ROW;
        unsigned char* sb = sa + BM * LDS_ROW;
#pragma unroll
        for (int it = 0; it < A_IT; ++it) {
          const int idx = tid + it * NT;
          const u32x4_t z = {0u, 0u, 0u, 0u};
          if (A_CH % NT == 0 || idx < A_CH)
            *(u32x4_t*)(sa + (idx / CPR) * LDS_ROW + (idx % CPR) * 16) = ((okm >> it) & 1u) ? ra[it] : z;
        }
#pragma unroll
        for (int it = 0; it < B_IT; ++it) {
          const int idx = tid + it * NT;
          if (B_CH % NT == 0 || idx < B_CH) *(u32x4_t*)(sb + (idx / CPR) * LDS_ROW + (idx % CPR) * 16) = rb[it];
        }
      };
      auto compute = [&](int stage) {
        const unsigned char* sa = smem + stage * (BM + BN) * LDS_ROW;
        const unsigned char* sb = sa + BM * LDS_ROW;
#pragma unroll
        for (int kg = 0; kg < KG; ++kg) {
          u32x4_t fa[TM], fb[TN];
#pragma unroll
          for (int i = 0; i < TM; ++i)
            fa[i] = *(const u32x4_t*)(sa + (wave_m * WM + i * 32 + l31) * LDS_ROW + kg * 32 + lhalf * 16);
#pragma unroll
          for (int j = 0; j < TN; ++j)
            fb[j] = *(const u32x4_t*)(sb + (wave_n * WN + j * 32 + l31) * LDS_ROW + kg * 32 + lhalf * 16);
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) {
              if constexpr (sizeof(T) == 2) {
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fa[i]),
                                                                    __builtin_bit_cast(bf16x8_t, fb[j]), acc[i][j], 0, 0, 0);
              } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                  acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fa[i][e]), __uint_as_float(fb[j][e]),
                                                                   acc[i][j], 0, 0, 0);
              }
            }
        }
      };

#pragma unroll
      for (int d = 0; d < D; ++d) {
        okm_[d] = 0;
        if (d < nsteps) load_global(d, ra[d], rb[d], okm_[d]);     // (uniform; the loader's position advances step by step)
      }
      for (int step0 = 0; step0 < nsteps; step0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
          const int step = step0 + d;
          if (step < nsteps) {                                     // (uniform)
            // stage d % 2 was last read by step - 2, which every wavefront finished before the barrier of step - 1
            store_lds(d & 1, ra[d], rb[d], okm_[d]);
            if (step + D < nsteps) load_global(step + D, ra[d], rb[d], okm_[d]);
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);    // keep the requests ahead of the MFMA block
            compute(d & 1);
          }
        }
      }
      __syncthreads();                            // the epilogue's staging aliases the operand stages

      // ---- epilogue: the rest of the linked chain ------------------------------------------------
      // Phase 1: raw accumulators to LDS (aliases the operand stages; the loop above ended with a barrier).
      // Accumulator element e of lane l in a 32x32 tile: row = (e/4)*8 + (l/32)*4 + e%4, column = l%32.
      float* stg = (float*)smem;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int col = wave_n * WN + j * 32 + l31;
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int row = wave_m * WM + i * 32 + (e >> 2) * 8 + lhalf * 4 + (e & 3);
            stg[row * SP + col] = acc[i][j][e];
          }
        }
      __syncthreads();

      // Phase 2: each thread finishes CE consecutive channels of one output element: scale/shift, shortcut,
      // ReLU, pooling over the rows of its window, then one 16-byte store into the consumer's buffer.
      if (MODE == M_FLAT && partial) {
        // reduction split: raw fp32 partial sums go to part[zsplit][m][k]; splitk_finish adds the shares in a fixed
        // order and runs the rest of the chain
        const int cg = tid % CG, col0 = cg * CE;
        for (int idx = tid; idx < BM * CG; idx += NT) {
          const int q = idx / CG, m = tile_m * BM + q;
          if (m >= a.M_total) break;
          float* dst = a.part + ((long long)zsplit * a.M_total + m) * a.part_ld + tile_n * BN + col0;
          const float* sp = stg + q * SP + col0;
#pragma unroll
          for (int e = 0; e < CE; e += 4) *(f32x4_t*)(dst + e) = *(const f32x4_t*)(sp + e);
        }
      } else if (MODE != M_GAP) {
        const int nq = MODE == M_FLAT ? BM : MODE == M_ZIGZAG ? BM / 4 : a.pph * a.ppw;
        // NT is a multiple of CG, so a thread keeps its channel group over all its output elements: the
        // folded scale / shift are loaded once, outside the loop (the arrays are padded to the tile)
        static_assert(NT % CG == 0, "channel group must be loop-invariant per thread");
        const int cg = tid % CG, col0 = cg * CE, k0 = tile_n * BN + col0;
        float sc[CE], sh[CE];
        *(f32x4_t*)&sc[0] = *(const f32x4_t*)(a.scale + k0);
        *(f32x4_t*)&sh[0] = *(const f32x4_t*)(a.shift + k0);
        if (CE == 8) {
          *(f32x4_t*)&sc[4] = *(const f32x4_t*)(a.scale + k0 + 4);
          *(f32x4_t*)&sh[4] = *(const f32x4_t*)(a.shift + k0 + 4);
        }
        for (int idx = tid; idx < nq * CG; idx += NT) {
          const int q = idx / CG;
          if (k0 >= a.K) break;
          long long obase, rb_ = 0;
          float v[CE];
          if (MODE == M_FLAT) {
            const int m = tile_m * BM + q;
            if (m >= a.M_total) continue;
            const int n = m / OHW, p = m - n * OHW;
            obase = (long long)n * a.out_sN + (long long)p * a.out_sP;
            rb_ = (long long)n * a.res_sN + (long long)p * a.res_sP;
            const float* sp = stg + q * SP + col0;
#pragma unroll
            for (int e = 0; e < CE; e += 4) *(f32x4_t*)&v[e] = *(const f32x4_t*)(sp + e);
#pragma unroll
            for (int e = 0; e < CE; ++e) v[e] = v[e] * sc[e] + sh[e];
            if (a.has_res) {
              if (a.vec_res) {
                float r[CE];
                tr::unpack(*(const u32x4_t*)((const T*)a.res + rb_ + k0), r);
#pragma unroll
                for (int e = 0; e < CE; ++e) v[e] += r[e];
              } else {
#pragma unroll
                for (int e = 0; e < CE; ++e) if (k0 + e < a.K) v[e] += tr::ld(a.res, rb_ + k0 + e);
              }
            }
            if (a.relu) {
#pragma unroll
              for (int e = 0; e < CE; ++e) v[e] = fmx(v[e], 0.f);
            }
          } else if (MODE == M_ZIGZAG) {
            const int wdx = ((tile_m * BM) >> 2) + q;
            if (wdx >= (a.M_total >> 2)) continue;
            const int PHW = a.PH * a.PW;
            const int n = wdx / PHW, pq = wdx - n * PHW;
            obase = (long long)n * a.out_sN + (long long)pq * a.out_sP;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              float u[CE];
              const float* sp = stg + (4 * q + j) * SP + col0;
#pragma unroll
              for (int e = 0; e < CE; e += 4) *(f32x4_t*)&u[e] = *(const f32x4_t*)(sp + e);
#pragma unroll
              for (int e = 0; e < CE; ++e) {
                float x = u[e] * sc[e] + sh[e];
                if (a.relu) x = fmx(x, 0.f);
                v[e] = j == 0 ? x : (a.pool == POOL_MAX ? fmx_raw(v[e], x) : v[e] + x);
              }
            }
            if (a.pool == POOL_AVG) {
#pragma unroll
              for (int e = 0; e < CE; ++e) v[e] *= 0.25f;
            }
          } else {  // M_PATCH
            const int qy = q / a.ppw, qx = q - qy * a.ppw;
            const int gy = py * a.pph + qy, gx = px * a.ppw + qx;
            if (gy >= a.PH || gx >= a.PW) continue;
            obase = (long long)img * a.out_sN + (long long)(gy * a.PW + gx) * a.out_sP;
            float mx[CE], sum[CE];
#pragma unroll
            for (int e = 0; e < CE; ++e) { mx[e] = -INFINITY; sum[e] = 0.f; }
            int cnt = 0, cntp = 0;
            for (int r = 0; r < a.pk; ++r)
              for (int s = 0; s < a.pk; ++s) {
                const int cy = qy * a.ps + r, cx = qx * a.ps + s;
                const int oh = oy0 + cy, ow = ox0 + cx;
                if (oh < a.OH + a.pp && ow < a.OW + a.pp) ++cntp;
                if (oh < 0 || oh >= a.OH || ow < 0 || ow >= a.OW) continue;
                float u[CE];
                const float* sp = stg + (cy * a.patch_w + cx) * SP + col0;
#pragma unroll
                for (int e = 0; e < CE; e += 4) *(f32x4_t*)&u[e] = *(const f32x4_t*)(sp + e);
#pragma unroll
                for (int e = 0; e < CE; ++e) {
                  float x = u[e] * sc[e] + sh[e];
                  if (a.relu) x = fmx(x, 0.f);
                  mx[e] = fmx_raw(mx[e], x); sum[e] += x;
                }
                ++cnt;
              }
            const float inv = 1.f / (float)(a.cip ? cntp : cnt);
#pragma unroll
            for (int e = 0; e < CE; ++e) v[e] = a.pool == POOL_MAX ? mx[e] : sum[e] * inv;
          }
          if (MODE == M_FLAT && a.ileave) {
            // two-group channel shuffle of concat(this chain, other part) done by the store: the finished channels and
            // the other part's channels of the same pixel alternate, 2 CE channels = two 16-byte stores
            ileave_store<T>((T*)a.out + obase + 2 * k0, tr::pack(v), *(const u32x4_t*)((const T*)a.res + rb_ + k0), a.ileave == 1);
          } else if (a.vec_out) {
            *(u32x4_t*)((T*)a.out + obase + k0) = tr::pack(v);
          } else {
#pragma unroll
            for (int e = 0; e < CE; ++e) {
              if (k0 + e >= a.K) continue;
              const long long o = obase + (long long)(k0 + e) * a.out_sK;
              if (a.out_f32) ((float*)a.out)[o] = v[e]; else tr::st(a.out, o, v[e]);
            }
          }
        }
      } else {
        // global average: thread (part, col) adds the rows part, part + NT/BN, ... of its column, in row order
        const int col = tid % BN, part = tid / BN;
        const int k = tile_n * BN + col;
        const float sc = a.scale[k], sh = a.shift[k];
        for (int row = part; row < BM; row += NT / BN) {
          if (mc * BM + row >= OHW) break;
          float x = stg[row * SP + col] * sc + sh;
          if (a.has_res && k < a.K) x += tr::ld(a.res, (long long)img * a.res_sN + (long long)(mc * BM + row) * a.res_sP + k);
          if (a.relu) x = fmx(x, 0.f);
          gsum += x;
        }
      }
      __syncthreads();                                             // staging is reused as operand stage 0
    }  // chunks

    if (MODE == M_GAP) {
      float* red = (float*)smem;                                   // [NT/BN][BN], fixed-order final sum
      red[tid] = gsum;                                             // tid == part * BN + col
      __syncthreads();
      if (tid < BN) {
        const int k = tile_n * BN + tid;
        if (k < a.K) {
          float s = 0.f;
          for (int part = 0; part < NT / BN; ++part) s += red[part * BN + tid];
          s /= (float)OHW;
          const long long o = (long long)img * a.out_sN + (long long)k * a.out_sK;
          if (a.out_f32) ((float*)a.out)[o] = s; else tr::st(a.out, o, s);
        }
      }
      __syncthreads();
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Dense 3x3 / stride 1 / pad 1 convolution chain with the input halo staged on chip
// ---------------------------------------------------------------------------------------------
// The im2col gather of conv_kernel re-reads every input pixel nine times through L2 and re-writes it nine
// times into LDS; LDS writes (~75 B/clk/CU) and L2->CU traffic (~45 B/clk/CU) then cost as much as the MFMA
// work.  Here a workgroup owns a TH x TW block of output pixels (256 GEMM rows) x BN (128 or 64) output channels,
// loads the (TH+2) x (TW+2) input patch of one 64-element channel chunk ONCE, and runs the nine taps out of that
// patch (the fragment address of a row only shifts by the tap offset).  This is the GPU form of the paper's halo
// replication (Section 4.1, last paragraph): neighbouring tiles hold their own copy of the boundary rows and
// columns instead of looking back.  Images are stacked with their padding rows (row q = n*(H+2) + oh), so a
// tile may span two images and small maps still fill the 256 rows; rows with oh >= H are dummies.
//
// Workgroups are persistent (one per compute unit) and walk their tiles as one long sequence of channel chunks:
// during the last chunk of a tile the first patch and the first two weight steps of the NEXT tile are already
// on their way, so a tile boundary costs the epilogue only.  The GEMM is computed transposed (accumulator rows =
// output channels, columns = pixels): a lane then owns 4 consecutive channels of one pixel, the 2x2 pooling
// window of the zig-zag enumeration is 4 neighbouring lanes (reduced with DPP quad permutes), and the finished
// values go through LDS once, already in the output type, to be stored as whole 16-byte channel groups.
constexpr int V2_BM = 256, V2_PPMAX = kHaloPatchMax;
// wavefronts per workgroup: 8 (4 x 2 of 64 pixels x BN/2 channels).  4 wavefronts of 64 x BN (a quarter fewer LDS
// fragment reads per MFMA) were measured 20-60 % slower: one wavefront per SIMD cannot hide the fragment-read latency.
constexpr int V2_NW = 8;
constexpr int V2_NT = 64 * V2_NW;
// The LDS writes that publish a later step follow the MFMAs of a tap (interleaved after the first k-group they were
// measured 4-7 % slower on VGG-16 layers, batch 32, bf16: the writes then delay the fragment reads).
// Weight stages in LDS: step s is read from stage s % 3 while step s + 2 is written to stage (s + 2) % 3, so stage
// (s + 1) % 3 is already visible during step s and the first fragments of step s + 1 are fetched before the barrier
// that ends step s: the MFMAs of a step start right after the barrier instead of after an LDS round trip.
constexpr int V2_WST = 3;
// how many k-groups ahead of the MFMAs the fragments are fetched from LDS
constexpr int V2_FD = 1;
// 1: the global loads and LDS writes of a step are spread between its MFMAs; 0: loads before, writes behind them
constexpr int V2_SPREAD = 1;
constexpr int V2_ABYTES = V2_PPMAX * LDS_ROW;
__host__ __device__ constexpr int v2_lds(int bn) { return 2 * V2_ABYTES + V2_WST * bn * LDS_ROW; }   // operand buffers
__host__ __device__ constexpr int v2_lds_total(int bn) { return v2_lds(bn) + 2 * bn * 4 + V2_BM * 12; }  // + scale / shift of the tile, + the row tables
// passes of the epilogue staging (rows of the tile per pass = rows / passes), sized to one patch buffer
__host__ __device__ constexpr int v2_passes(int rows, int pitch) {
  return rows * pitch <= V2_ABYTES ? 1 : (rows / 2) * pitch <= V2_ABYTES ? 2 : 4;
}

template <int CTRL>
__device__ __forceinline__ float quad_perm(float v) {
  return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xf, 0xf, true));
}
// One step of the reduction over a lane quad in ONE instruction: v (op) v of the lane that the quad permutation names
// (the DPP modifier on the arithmetic instruction instead of a separate lane move).  SWAP1 = lanes [1,0,3,2], else [2,3,0,1].
// The two wait states a DPP read needs after a VALU write of its source are inside the asm, where the compiler's hazard
// recogniser does not look.
template <bool SWAP1>
__device__ __forceinline__ float quad_max(float v) {
  float r;
  if (SWAP1) asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(v));
  else asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(v));
  return r;
}
template <bool SWAP1>
__device__ __forceinline__ float quad_add(float v) {
  float r;
  if (SWAP1) asm("s_nop 1\n\tv_add_f32_dpp %0, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(v));
  else asm("s_nop 1\n\tv_add_f32_dpp %0, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(v));
  return r;
}

// PWID = row pitch of the staged patch in pixels (compile time, so that every tap is an immediate LDS offset).
// PWID = 0 selects the patch-linear form (pixel-major enumeration only): the pitch is TW + 2 at run time and GEMM row m
// IS patch position m, halo columns included (two junk rows per patch row, never stored).  The A fragments of every
// tap are then 32 consecutive LDS rows per half-wavefront, the one pattern `ds_read_b128` serves at 238 B/clk/CU
// (measured; any other row pattern runs at 127 B/clk/CU).  Measured on VGG-16 layers it is within +-3 % of the plain form
// (the junk rows cost what the faster reads gain) and 6 % faster on 14x14 maps; the tuner picks it where it wins.
// PART (pixel-major chains only): the reduction is split across workgroups as well (Section 4.2.2: a C split needs an
// additional reduction).  A work item is (pixel tile, channel tile, share z): share z covers the channel chunks
// [z * a.steps_per_split, (z + 1) * a.steps_per_split) and writes raw fp32 sums to a.part[z][pixel][channel]; the summing
// pass adds the shares in index order and runs the rest of the chain.  For maps so small that pixel x channel tiles
// leave most compute units idle (7x7 and 14x14 at batch 32).
template <typename T, int MODE, int PWID, int BN, bool PART = false>
__global__ __launch_bounds__(V2_NT) void conv3x3_kernel(const ConvArgs a) {
  using tr = Tr<T>;
  constexpr int CE = tr::CE, BKE = tr::BKE, ESZ = (int)sizeof(T);
  constexpr int BM = V2_BM, NTH = V2_NT;
  constexpr int WAVES_N = V2_NW / 4;                               // 4 x WAVES_N wavefronts of 64 pixels x WN channels
  constexpr int WN = BN / WAVES_N, TN = WN / 32;
  constexpr int A_IT = (V2_PPMAX * CPR + 2 * NTH - 1) / (2 * NTH) * 2;   // patch chunks per thread (an even count; the last may lie beyond the buffer)
  constexpr int B_IT = BN * CPR / NTH;                             // weight chunks per thread
  constexpr int BBYTES = BN * LDS_ROW;
  constexpr int CG = BN / CE;                                      // 16-byte channel groups per output row
  constexpr int SPB = BN * ESZ + 16;                               // staging row pitch in bytes
  constexpr int ROWS = MODE == M_FLAT ? BM : BM / 4;               // staged rows: pixels, or pooled windows
  // The finished tile is staged in the patch buffer that is free at the end of a tile; when the free weight stage can
  // take the rows that do not fit there (bf16, 128 channels: 192 + 64 rows), the whole tile is staged at once,
  // otherwise in NP passes of RPP rows.
  constexpr int R1 = ROWS * SPB <= V2_ABYTES ? ROWS : V2_ABYTES / SPB;   // rows staged in the patch buffer
  constexpr bool SPLIT_STG = R1 < ROWS && R1 > 0 && (ROWS - R1) * SPB <= BBYTES;
  constexpr int NP = SPLIT_STG ? 1 : v2_passes(ROWS, SPB), RPP = ROWS / NP;
  static_assert(MODE == M_FLAT || MODE == M_ZIGZAG, "row enumerations of the halo kernel");
  static_assert(A_IT % 2 == 0 && B_IT >= 1 && NTH % CG == 0, "loader shapes");
  static_assert((A_IT - 1) * NTH <= V2_PPMAX * CPR && A_IT >= 4, "only the last chunk of a thread may lie beyond the patch buffer");

  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
  const int l31 = lane & 31, lhalf = lane >> 5;
  // Which GEMM row (pixel) of a 32-row block this lane holds.  `ds_read_b128` serves a half-wavefront in two passes of 16
  // lanes: the lanes whose bits 2, 3, 4 have even parity, and those with odd parity (measured with 30 access patterns: 245
  // B/clk/CU when the 16 lanes of each pass read LDS rows that differ mod 16 at the 144-byte pitch, 127 otherwise).  The
  // two 16-pixel blocks of the enumerations below, whose pixels have 16 different residues each, are therefore dealt to
  // those two lane sets, lane quads kept whole (the pooling epilogue reduces over quads).
  const int lq = l31 >> 2;
  const int lp = (((0x96 >> lq) & 1) << 4) | ((lq >> 1) << 2) | (l31 & 3);

  constexpr bool PLIN = PWID == 0;
  static_assert(!PLIN || MODE == M_FLAT, "the patch-linear form exists for the pixel-major enumeration");
  const int PW_ = PLIN ? a.tw + 2 : PWID;                          // patch row pitch in pixels (a.tw + 2 <= PW_)
  const int PP = (a.th + 2) * PW_ + (PLIN ? 2 : 0), Hp = a.H + 2;  // (the last tap of the last junk rows reads 2 positions further)
  const int KS = PART ? a.ksplit : 1;                              // shares of the reduction
  const int nchunks = PART ? a.steps_per_split : a.C / BKE;        // channel chunks of one work item
  static_assert(!PART || MODE == M_FLAT, "the reduction split exists for pixel-major chains");

  // ---- this workgroup's tiles ---------------------------------------------------------------------
  // Workgroups are dealt round-robin to the XCDs; each XCD owns a contiguous, balanced range of pixel tiles and
  // walks it once per output-channel tile, so its workgroups share one weight slice in their L2 and neighbouring
  // pixel tiles share their input halo.
  // (with at least 8 workgroups, the usual case, the divisions by the XCD count are shifts; every scalar division in this
  // set-up is a long dependent chain in front of the kernel's first load)
  const int G = gridDim.x;
  const bool full = G >= NUM_XCD;
  const int nx = full ? NUM_XCD : G;
  const int xcd = full ? (int)(blockIdx.x & (NUM_XCD - 1)) : (int)blockIdx.x;
  const int wgs = full ? (G - xcd + NUM_XCD - 1) / NUM_XCD : 1;    // workgroups of this XCD
  const int m0 = full ? xcd * a.tiles_m / NUM_XCD : xcd * a.tiles_m / nx;
  const int mlen = (full ? (xcd + 1) * a.tiles_m / NUM_XCD : (xcd + 1) * a.tiles_m / nx) - m0;
  const int TNX = a.tiles_n * KS;                                  // channel tiles x reduction shares: one index
  const int ntl = mlen * TNX;                                      // work items of this XCD
  // Order of an XCD's tiles: groups of `mg` pixel tiles, each group once per output-channel tile before the next group.
  // With a group as large as the XCD's range this is one sweep per channel tile (one weight slice live in the L2 at a
  // time); a group that the XCD's workgroups cover in one or two rounds reads its input patches while they are still
  // in the L2 instead of once per channel tile.
  const int mg = a.halo_mgroup < mlen ? a.halo_mgroup : mlen;
  auto tile_of = [&](int l, int& tile_m, int& tile_n) __attribute__((always_inline)) {
    const int per = mg * TNX, grp = l / per, r = l - grp * per;
    const int left = mlen - grp * mg, glen = left < mg ? left : mg;   // the last group of the range may be short
    tile_n = r / glen;
    tile_m = m0 + grp * mg + (r - tile_n * glen);
  };
  int li = full ? (int)(blockIdx.x / NUM_XCD) : 0;
  if (li >= ntl) return;                                           // uniform per workgroup
  // A tile of the workgroup's sequence, decoded once (three uniform divisions) and kept for everything that needs it:
  // loads, weights, epilogue tables, epilogue
  struct Tile { int tile_n, q0, x0, n0, r0, z; };
  auto decode = [&](int l) __attribute__((always_inline)) -> Tile {
    int tile_m, tile_n;
    tile_of(l, tile_m, tile_n);
    const int z = PART ? tile_n % KS : 0;                          // (tile_of hands back the combined index)
    if (PART) tile_n /= KS;
    const int tyi = tile_m / a.tiles_x;
    const int q0 = tyi * a.th, n0 = q0 / Hp;
    return Tile{tile_n, q0, (tile_m - tyi * a.tiles_x) * a.tw, n0, q0 - n0 * Hp, z};
  };
  // image and row of stacked row t.q0 + y: compares as long as a tile spans at most four images
  const bool few = a.th + 2 <= 3 * Hp;
  auto image_row = [&](const Tile& t, int y, int& n, int& row) __attribute__((always_inline)) {
    const int rel = t.r0 + y;
    const int k = few ? (rel >= Hp ? 1 : 0) + (rel >= 2 * Hp ? 1 : 0) + (rel >= 3 * Hp ? 1 : 0) : rel / Hp;
    n = t.n0 + k; row = rel - k * Hp;
  };
  Tile tcur = decode(li), tnext = tcur;

  // ---- what this thread loads for a tile: 6 chunks of the input patch, B_IT chunks of the weight tile ------
  int aoff[A_IT];
  unsigned aok = 0;
  // byte offset of this thread's first weight chunk in the packed weights, for this tile and for the next one; its
  // other chunks lie NTH / 8 rows further each
  int wrow = 0, wnext = 0;
  const int wstride = (NTH / CPR) * a.Kred_pad * ESZ;
  auto patch_addr = [&](const Tile& t) __attribute__((always_inline)) {
    // image and row of a stacked row: one division per tile (uniform, in decode()), then compares per chunk as long as a
    // patch spans at most four images (this runs between the MFMA streams of two tiles: with one channel chunk per tile it
    // was a tenth of the tile's time when every chunk divided)
    const int n0 = t.n0, r0 = t.r0, x0 = t.x0;
    const int sN = (int)a.in_sN, sH = (int)a.in_sH, sW = (int)a.in_sW;   // (N * in_sN < 2^31 is checked by the host)
    aok = 0;
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
      const int idx = tid + it * NTH;
      const int pp = idx / CPR, c8 = idx % CPR;
      const int pr = pp / PW_, pc = pp - pr * PW_;
      const int rel = r0 + pr;
      const int k = few ? (rel >= Hp ? 1 : 0) + (rel >= 2 * Hp ? 1 : 0) + (rel >= 3 * Hp ? 1 : 0) : rel / Hp;
      const int n = n0 + k, ih = rel - k * Hp - 1, iw = x0 - 1 + pc;
      const bool ok = pp < PP && n < a.N && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
      aoff[it] = (ok ? n * sN + ih * sH + iw * sW + c8 * CE : c8 * CE) + (PART ? t.z * nchunks * BKE : 0);
      aok |= (ok ? 1u : 0u) << it;
    }
  };
  auto weight_addr = [&](const Tile& t) __attribute__((always_inline)) -> int {
    return ((t.tile_n * BN + tid / CPR) * a.Kred_pad + (tid % CPR) * CE) * ESZ + (PART ? t.z * nchunks * 9 * ROWB : 0);
  };

  // ---- which pixel of the tile a GEMM row is ---------------------------------------------------------------
  // A ds_read_b128 pass of 16 lanes is conflict-free when their LDS rows differ mod 16 (row pitch 144 B).
  // A pixel (ty, tx) sits in patch row ty * PWID + tx = 2 * ty + tx (mod 16), so the rows of a tile are enumerated in
  // blocks whose 16 pixels have 16 different residues: 8 rows x 2 columns for the pixel-major enumeration, 4
  // vertically adjacent 2x2 windows for the zig-zag one (a window covers 4 consecutive residues).  Rows left over
  // when TH is not a multiple of 8 follow in plain order.  Any enumeration is legal: every pixel carries its own
  // output address.
  // (pitch = 2 mod 8: rows ty = 0 .. 7 then start at 8 different even residues mod 16, with pitch 18 and 34 in order,
  // with pitch 10 permuted; a 2x2 window of the zig-zag enumeration covers 4 residues and 4 stacked windows all 16)
  static_assert(PLIN || PWID % 8 == 2, "the conflict-free enumeration assumes patch pitch = 2 mod 8");
  auto flat_px = [&](int m, int& ty, int& tx) __attribute__((always_inline)) {
    if (PLIN) { ty = m / PW_; tx = m - ty * PW_; return; }
    const int nbx = a.tw >> 1, rows8 = (a.tw & 1) ? 0 : (a.th >> 3) * 8, full = rows8 * a.tw;
    if (m < full) {
      const int b = m >> 4, i = m & 15, by = b / nbx, bx = b - by * nbx;
      ty = by * 8 + (i >> 1); tx = bx * 2 + (i & 1);
    } else {
      const int r = m - full, y = r / a.tw;
      ty = rows8 + y; tx = r - y * a.tw;
    }
  };
  auto zz_win = [&](int w, int& wy, int& wx) __attribute__((always_inline)) {
    const int hw = a.tw >> 1, rows4 = (a.th >> 3) * 4, full = rows4 * hw;
    if (w < full) {
      const int g = w / (4 * hw), r = w - g * 4 * hw;
      wx = r >> 2; wy = g * 4 + (r & 3);
    } else {
      const int r = w - full, y = r / hw;
      wy = rows4 + y; wx = r - y * hw;
    }
  };

  // which pixel (or pooling window) of the tile each staged row is: the same for every tile, so it is worked out once
  // (the integer divisions of the enumeration would otherwise be paid per stored channel group)
  int* s_rowpos = (int*)(smem + v2_lds(BN) + 2 * BN * 4);          // (filled at the pipeline start, beside its first loads)

  // ---- fragment addresses of this lane's rows (pixels of the tile); the same for every tile (worked out at the
  // pipeline start, while its first loads are on their way) --------------
  int abase[2], bbase[TN];

  f32x16_t acc[2][TN];
  constexpr int A_HALF = A_IT / 2;
  u32x4_t pa[A_HALF], rb0[B_IT], rb1[B_IT];

  // the patch of a channel chunk travels in two halves of 3 chunks per thread (12 staging registers)
  auto load_patch = [&](int c, int half) {
#pragma unroll
    for (int it = 0; it < A_HALF; ++it) pa[it] = *(const u32x4_t*)((const T*)a.in + aoff[half * A_HALF + it] + c);
  };
  auto store_patch = [&](int buf, int half) {
    unsigned char* sa = smem + buf * V2_ABYTES;
    const u32x4_t z = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int it = 0; it < A_HALF; ++it) {
      const int g = half * A_HALF + it;
      int idx = tid + g * NTH;
      u32x4_t v = ((aok >> g) & 1u) ? pa[it] : z;
      if ((g + 1) * NTH > V2_PPMAX * CPR) {
        // the last chunks of some threads lie beyond the buffer: those threads write their previous chunk once more
        // (same address, same value) instead of branching around the store
        const bool in = idx < V2_PPMAX * CPR;
        const u32x4_t vp = ((aok >> (g - 1)) & 1u) ? pa[it - 1] : z;
        idx = in ? idx : idx - NTH;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = in ? v[e] : vp[e];
      }
      *(u32x4_t*)(sa + (idx / CPR) * LDS_ROW + (idx % CPR) * 16) = v;
    }
  };
  auto load_w = [&](int step, u32x4_t* rb) {
#pragma unroll
    for (int it = 0; it < B_IT; ++it) rb[it] = *(const u32x4_t*)((const unsigned char*)a.w + wrow + it * wstride + step * ROWB);
  };
  auto store_w = [&](int stage, const u32x4_t* rb) {
    unsigned char* sb = smem + 2 * V2_ABYTES + stage * BBYTES;
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
      const int idx = tid + it * NTH;
      *(u32x4_t*)(sb + (idx / CPR) * LDS_ROW + (idx % CPR) * 16) = rb[it];
    }
  };
  // one tap of one channel chunk: 4 k-groups, fragments of k-group g + V2_FD are fetched before the MFMAs of g; the
  // fragments of the first k-groups were fetched during the previous step, and the last k-groups fetch those of the next
  // step (`nsa`, `nsb`: its patch position and weight stage, both published at least one barrier ago)
  u32x4_t fa[V2_FD + 1][2], fb[V2_FD + 1][TN];
  static_assert((9 * KG) % (V2_FD + 1) == 0, "the fragment slots rotate per k-group and must line up across chunks");
  auto fetch = [&](int slot, const unsigned char* sa, const unsigned char* sb, int kg) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < 2; ++i) fa[slot][i] = *(const u32x4_t*)(sa + abase[i] + kg * 32);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[slot][j] = *(const u32x4_t*)(sb + bbase[j] + kg * 32);
  };
  // `tap` is a constant of the unrolled tap loop: the slot of k-group g of tap t is (t * KG + g) % (V2_FD + 1)
  auto compute = [&](int tap, const unsigned char* sa, const unsigned char* sb, const unsigned char* nsa, const unsigned char* nsb) {
#pragma unroll
    for (int kg = 0; kg < KG; ++kg) {
      const int cur = (tap * KG + kg) % (V2_FD + 1), nxt = (tap * KG + kg + V2_FD) % (V2_FD + 1);
      if (kg + V2_FD < KG) fetch(nxt, sa, sb, kg + V2_FD);
      else fetch(nxt, nsa, nsb, kg + V2_FD - KG);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          // operands swapped: accumulator rows = channels of block j, columns = pixels of block i
          if constexpr (sizeof(T) == 2) {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fb[cur][j]),
                                                                __builtin_bit_cast(bf16x8_t, fa[cur][i]), acc[i][j], 0, 0, 0);
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fb[cur][j][e]), __uint_as_float(fa[cur][i][e]),
                                                               acc[i][j], 0, 0, 0);
          }
        }
    }
  };
  // The schedule wanted for one tap (0x100 = LDS read, 0x200 = LDS write, 0x020 = global load, 0x008 = MFMA): the
  // fragments of the following k-group are in flight while the MFMAs of a k-group issue; the global loads of the step
  // are spread between the first MFMAs and the LDS writes that publish a later step between the last ones, so that no
  // wavefront spends a stretch of the step issuing memory instructions with its MFMA pipe idle (an MFMA occupies the
  // pipe for 32 cycles and the wavefront is free to issue other instructions meanwhile).  Without the directives the
  // scheduler serialises read -> wait -> MFMA.
  auto tap_schedule = [&](bool patch_loads, bool patch_writes) {
    constexpr int NM = (sizeof(T) == 2 ? 2 : 8) * TN;              // MFMAs per k-group
    static_assert(NM >= 2, "the memory instructions go behind the first two MFMAs of a k-group");
#pragma unroll
    for (int kg = 0; kg < KG; ++kg) {
      __builtin_amdgcn_sched_group_barrier(0x100, 2 + TN, 0);
      if (V2_SPREAD && kg == 0) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (patch_loads) __builtin_amdgcn_sched_group_barrier(0x020, (B_IT + A_HALF + 1) / 2, 0);
        else __builtin_amdgcn_sched_group_barrier(0x020, (B_IT + 1) / 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (patch_loads) __builtin_amdgcn_sched_group_barrier(0x020, (B_IT + A_HALF) / 2, 0);
        else if (B_IT / 2 > 0) __builtin_amdgcn_sched_group_barrier(0x020, B_IT / 2, 0);
        if (NM > 2) __builtin_amdgcn_sched_group_barrier(0x008, NM - 2, 0);
      } else if (V2_SPREAD && kg == KG - 1) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (patch_writes) __builtin_amdgcn_sched_group_barrier(0x200, (B_IT + A_HALF + 1) / 2, 0);
        else __builtin_amdgcn_sched_group_barrier(0x200, (B_IT + 1) / 2, 0);
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        if (patch_writes) __builtin_amdgcn_sched_group_barrier(0x200, (B_IT + A_HALF) / 2, 0);
        else if (B_IT / 2 > 0) __builtin_amdgcn_sched_group_barrier(0x200, B_IT / 2, 0);
        if (NM > 2) __builtin_amdgcn_sched_group_barrier(0x008, NM - 2, 0);
      } else {
        __builtin_amdgcn_sched_group_barrier(0x008, NM, 0);
      }
    }
  };
  int aff_tile_n = -1;                                             // channel tile whose scale / shift are in LDS
  // What the epilogue of tile `l` reads from LDS, written during the tile's last chunk so that the barriers of that
  // chunk's taps publish it and the integer division per row is paid beside the MFMAs of the chunk, not between two tiles.
  auto epilogue_tables = [&](const Tile& t) __attribute__((always_inline)) {
    const int tile_n = t.tile_n, x0 = t.x0;
    // this tile's folded scale / shift, shared through LDS (every lane needs 32 of the BN values of each)
    float* s_aff = (float*)(smem + v2_lds(BN));
    if (tile_n != aff_tile_n) {   // a workgroup walks pixel tiles within a channel tile: reloaded only when that changes
      if (tid < 2 * BN) s_aff[tid] = tid < BN ? a.scale[tile_n * BN + tid] : a.shift[tile_n * BN + tid - BN];
      aff_tile_n = tile_n;
    }
    // where each staged row goes in the output (element offset of its channel 0; -1 = not an output of this tile)
    long long* s_rowoff = (long long*)(smem + v2_lds(BN) + 2 * BN * 4 + V2_BM * 4);
    for (int q = tid; q < ROWS; q += NTH) {
      const int pos = s_rowpos[q];
      long long ob = -1;
      if (pos >= 0) {
        const int y = pos >> 16, x = pos & 0xffff;
        int n, oh;
        image_row(t, MODE == M_FLAT ? y : 2 * y, n, oh);
        const int ow = x0 + (MODE == M_FLAT ? x : 2 * x);
        if (n < a.N && oh < a.H && ow < a.W)
          ob = (long long)n * a.out_sN + (MODE == M_FLAT ? (long long)(oh * a.OW + ow) : (long long)((oh >> 1) * a.PW + (ow >> 1))) * a.out_sP;
      }
      s_rowoff[q] = ob;
    }
  };
  // Nine statically unrolled taps of channel chunk cc.  PAR = parity of the chunk in the workgroup's whole chunk
  // sequence: it selects the patch buffer, and (9 steps per chunk) the register set of tap 0; the weight stage of a tap
  // is tap % 3 in every chunk.
  // `last`: the chunk after this one belongs to the next tile (aoff / aok / wnext already describe that tile).
  auto chunk_body = [&](int cc, bool last, auto par) {
    constexpr int PAR = decltype(par)::value;
    const int step0 = cc * 9;
    const int cnext = last ? 0 : (cc + 1) * BKE;
    unsigned char* const sw = smem + 2 * V2_ABYTES;
#pragma unroll
    for (int tap = 0; tap < 9; ++tap) {
      const int sp = (PAR + tap) & 1;                              // register set of this step
      u32x4_t* rb = sp == 0 ? rb0 : rb1;
      if (tap < 6) load_w(step0 + tap + 3, rb);                    // weights of step + 3 ...
      else {
        // ... which for the last three taps of a tile are steps 0, 1, 2 of the next tile
#pragma unroll
        for (int it = 0; it < B_IT; ++it) {
          const int src = (last ? wnext + (tap - 6) * ROWB : wrow + (step0 + tap + 3) * ROWB) + it * wstride;
          rb[it] = *(const u32x4_t*)((const unsigned char*)a.w + src);
        }
      }
      if (tap == 0) load_patch(cnext, 0);                          // next chunk's patch: half 0 in flight over taps 0-3,
      if (tap == 4) load_patch(cnext, 1);                          // half 1 over taps 4-7
      if (!V2_SPREAD) __builtin_amdgcn_sched_barrier(0);           // keep the prefetch loads ahead of the MFMA block
      const int tapoff = ((tap / 3) * PW_ + tap % 3) * LDS_ROW, ntapoff = (((tap + 1) / 3) * PW_ + (tap + 1) % 3) * LDS_ROW;
      compute(tap, smem + PAR * V2_ABYTES + tapoff, sw + (tap % 3) * BBYTES,
              tap < 8 ? smem + PAR * V2_ABYTES + ntapoff : smem + (PAR ^ 1) * V2_ABYTES, sw + ((tap + 1) % 3) * BBYTES);
      store_w((tap + 2) % 3, sp == 0 ? rb1 : rb0);                 // publish step + 2 (loaded during the previous step)
      if (tap == 3) store_patch(PAR ^ 1, 0);
      if (tap == 7) store_patch(PAR ^ 1, 1);                       // (complete one barrier before tap 8 fetches from it)
      tap_schedule(tap == 0 || tap == 4, tap == 3 || tap == 7);
      __builtin_amdgcn_sched_barrier(0);
      __syncthreads();
      // the tables of this tile's epilogue: after a barrier that every wavefront reaches only when it has finished the
      // previous tile's epilogue (which has no barrier of its own), and eight barriers before they are read
      if (tap == 0 && last) epilogue_tables(tcur);
    }
  };

  // ---- pipeline start: chunk 0, weight steps 0, 1 (in LDS) and 2 (in registers), first fragments of the first tile ----
  // Both halves of the first patch and the first two weight steps are requested together (one memory round trip, from
  // memory nobody has touched yet, instead of two), and the row table is worked out while they are on their way.
  patch_addr(tcur);
  wrow = weight_addr(tcur);
  load_patch(0, 0);
  u32x4_t pb[A_HALF];
#pragma unroll
  for (int it = 0; it < A_HALF; ++it) pb[it] = *(const u32x4_t*)((const T*)a.in + aoff[A_HALF + it]);   // = load_patch(0, 1)
  load_w(0, rb0);
  load_w(1, rb1);
  for (int q = tid; q < ROWS; q += NTH) {
    int y, x;
    if (MODE == M_FLAT) flat_px(q, y, x); else zz_win(q, y, x);
    const bool ok = MODE == M_FLAT ? (y < a.th && x < a.tw) : (2 * y < a.th && 2 * x < a.tw);
    s_rowpos[q] = ok ? (y << 16) | x : -1;
  }
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int m = wave_m * 64 + i * 32 + lp;
    int ty, tx;
    if (MODE == M_FLAT) flat_px(m, ty, tx);
    else {
      int wy, wx;
      zz_win(m >> 2, wy, wx);
      ty = 2 * wy + ((m >> 1) & 1); tx = 2 * wx + (m & 1);
    }
    const bool ok = ty < a.th && tx < a.tw;
    abase[i] = (PLIN ? m : ok ? ty * PW_ + tx : 0) * LDS_ROW + lhalf * 16;
  }
#pragma unroll
  for (int j = 0; j < TN; ++j) bbase[j] = (wave_n * WN + j * 32 + l31) * LDS_ROW + lhalf * 16;
  store_patch(0, 0);
#pragma unroll
  for (int it = 0; it < A_HALF; ++it) pa[it] = pb[it];
  store_w(0, rb0);
  store_w(1, rb1);
  store_patch(0, 1);
  load_w(2, rb1);
  __syncthreads();
#pragma unroll
  for (int g = 0; g < V2_FD; ++g) fetch(g, smem, smem + 2 * V2_ABYTES, g);

#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // The chain's epilogue for the tile `li`, run after its last chunk (of parity PAR).
  auto epilogue = [&](auto par) {
    constexpr int PAR = decltype(par)::value;
    const int tile_n = tcur.tile_n, x0 = tcur.x0;
    // Every wavefront finishes and stores its own 64 pixels x WN channels: a row of its block holds whole 16-byte channel
    // groups, so the values pass through LDS only to change hands between the lanes of that wavefront (LDS serves a
    // wavefront's requests in order) and the epilogue has no barrier.  A pass stages 32 pixels (8 pooling windows) x at
    // most 128 bytes of channels per wavefront in the patch buffer of the chunk just finished, which nobody writes before
    // tap 3 of the next chunk, three barriers later; the other buffer holds the next tile's first patch.
    constexpr int JP = WN * ESZ <= 128 ? TN : 1;                   // 32-channel blocks per pass
    constexpr int RB = JP * 32 * ESZ;                              // bytes of channels per staged row
    constexpr int SPW = RB + (ESZ == 2 ? 8 : 16);                  // row pitch: 34 dwords (bf16) puts the 32 rows of an 8-byte store pass in 32 different bank pairs
    constexpr int PROWS = MODE == M_FLAT ? 32 : 8;                 // staged rows per pass
    static_assert(8 * 32 * SPW <= V2_ABYTES, "the per-wavefront staging areas must fit the free patch buffer");
    unsigned char* wstg = smem + PAR * V2_ABYTES + wave * (32 * SPW);
    // shortcut address of this lane's two pixels (rows outside the image read element 0)
    long long rbase[2] = {0, 0};
    if (MODE == M_FLAT && a.has_res) {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int m = wave_m * 64 + i * 32 + lp;
        int ty, tx;
        flat_px(m, ty, tx);
        int n, oh;
        image_row(tcur, ty < a.th ? ty : 0, n, oh);
        const int ow = x0 + tx;
        const bool ok = ty < a.th && n < a.N && oh < a.H && ow < a.W;
        rbase[i] = ok ? (long long)n * a.res_sN + (long long)(oh * a.OW + ow) * a.res_sP : 0;
      }
    }
    const float lo = a.relu ? 0.f : -3.4028235e38f;                // ReLU as a clamp: no branch per value
    // (the tile's scale / shift and the output offsets of its rows were put into LDS by epilogue_tables() after the first
    // tap of the tile's last chunk: eight barriers ago)
    const float* s_aff = (const float*)(smem + v2_lds(BN));
    const long long* s_rowoff = (const long long*)(smem + v2_lds(BN) + 2 * BN * 4 + V2_BM * 4);
    // a pass: the lanes finish their accumulators of pixel block i, channel blocks j0 .. j0 + JP - 1 (scale, shift,
    // shortcut, ReLU, pooling), stage them in the output type, and the wavefront stores the staged rows as whole groups.
    // RES / PMAX are compile-time copies of the chain's flags, so the channel groups of a lane run without branches.
    auto finish_store = [&](auto res_c, auto max_c) {
      constexpr bool RES = decltype(res_c)::value, PMAX = decltype(max_c)::value;
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j0 = 0; j0 < TN; j0 += JP) {
          const int m = wave_m * 64 + i * 32 + lp;
          const int srow = MODE == M_FLAT ? lp : (lp >> 2);
#pragma unroll
          for (int jj = 0; jj < JP; ++jj)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
              const int j = j0 + jj;
              const int cl = jj * 32 + g * 8 + lhalf * 4;          // channel within the staged row
              const int c = wave_n * WN + j * 32 + g * 8 + lhalf * 4, k0 = tile_n * BN + c;
              const f32x4_t sc = *(const f32x4_t*)(s_aff + c), sh = *(const f32x4_t*)(s_aff + BN + c);
              float y[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) y[e] = acc[i][j][4 * g + e] * sc[e] + sh[e];
              if constexpr (RES) {
                // rows outside the image and channel groups beyond K read a valid dummy address; they are never stored
                const long long ra = rbase[i] + (k0 < a.K ? k0 : 0);
                if constexpr (sizeof(T) == 2) {
                  const uint2 r = *(const uint2*)((const T*)a.res + ra);
                  y[0] += __uint_as_float(r.x << 16); y[1] += __uint_as_float(r.x & 0xffff0000u);
                  y[2] += __uint_as_float(r.y << 16); y[3] += __uint_as_float(r.y & 0xffff0000u);
                } else {
                  const f32x4_t r = *(const f32x4_t*)((const T*)a.res + ra);
#pragma unroll
                  for (int e = 0; e < 4; ++e) y[e] += r[e];
                }
              }
#pragma unroll
              for (int e = 0; e < 4; ++e) y[e] = fmx(y[e], lo);
              bool mine = true;                                    // does this lane hold the finished value?
              if (MODE == M_ZIGZAG) {
                // the window's four pixels are lanes 4w .. 4w+3: butterfly over the quad, lane j keeps group g == j
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                  y[e] = PMAX ? quad_max<true>(y[e]) : quad_add<true>(y[e]);              // with lanes [1,0,3,2]
                  y[e] = PMAX ? quad_max<false>(y[e]) : quad_add<false>(y[e]) * 0.25f;   // with lanes [2,3,0,1]
                }
                mine = (l31 & 3) == g;
              }
              if (mine) {
                if constexpr (sizeof(T) == 2) {
                  uint2 o;
                  o.x = f2bf2(y[0], y[1]);
                  o.y = f2bf2(y[2], y[3]);
                  *(uint2*)(wstg + srow * SPW + cl * 2) = o;
                } else {
                  // (stored through the type the read-back uses: nothing but program order keeps the two apart)
                  *(u32x4_t*)(wstg + srow * SPW + cl * 4) = u32x4_t{__float_as_uint(y[0]), __float_as_uint(y[1]), __float_as_uint(y[2]), __float_as_uint(y[3])};
                }
              }
            }
          // the wavefront's staged rows, one 16-byte channel group per lane and turn
          constexpr int G = RB / 16, NGW = PROWS * G / 64 > 0 ? PROWS * G / 64 : 1;
          const int qbase = MODE == M_FLAT ? wave_m * 64 + i * 32 : (wave_m * 64 + i * 32) / 4;
          long long ob[NGW];
          u32x4_t v[NGW];
#pragma unroll
          for (int u = 0; u < NGW; ++u) {
            const int idx = lane + u * 64;
            const bool in = idx < PROWS * G;
            const int r = in ? idx / G : 0, cg = idx % G;
            ob[u] = in ? s_rowoff[qbase + r] : -1;
            if constexpr (sizeof(T) == 2) {
              const uint2 lo8 = *(const uint2*)(wstg + r * SPW + cg * 16), hi8 = *(const uint2*)(wstg + r * SPW + cg * 16 + 8);
              v[u] = u32x4_t{lo8.x, lo8.y, hi8.x, hi8.y};
            } else {
              v[u] = *(const u32x4_t*)(wstg + r * SPW + cg * 16);
            }
          }
#pragma unroll
          for (int u = 0; u < NGW; ++u) {
            const int cg = (lane + u * 64) % G, k0 = tile_n * BN + wave_n * WN + j0 * 32 + cg * CE;
            if (ob[u] >= 0 && k0 < a.K) *(u32x4_t*)((T*)a.out + ob[u] + k0) = v[u];
          }
        }
    };
    using std::true_type; using std::false_type;
    if constexpr (PART) {
      // raw fp32 sums of this share: lane = pixel lp of block i, 4 consecutive channels per group; the row table holds
      // pixel * part_ld (the host sets the output strides to the partial buffer's)
      float* pz = a.part + (long long)tcur.z * a.M_total * a.part_ld;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const long long ob = s_rowoff[wave_m * 64 + i * 32 + lp];
        if (ob < 0) continue;
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int k0 = tile_n * BN + wave_n * WN + j * 32 + g * 8 + lhalf * 4;
            *(f32x4_t*)(pz + ob + k0) = f32x4_t{acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
          }
      }
    } else if (MODE == M_FLAT) {
      if (a.has_res) finish_store(true_type{}, false_type{});
      else finish_store(false_type{}, false_type{});
    } else {
      if (a.pool == POOL_MAX) finish_store(false_type{}, true_type{});
      else finish_store(false_type{}, false_type{});
    }
  };

  // One channel chunk of the workgroup's chunk sequence; returns true when the workgroup has finished its last tile.
  // The two parities alternate in straight-line code, so the accumulators never meet at a control-flow join.
  int cc = 0;
  auto advance = [&](auto par) -> bool {
    const bool last = cc == nchunks - 1;
    if (last) {
      const int lnext = li + wgs < ntl ? li + wgs : li;            // after the last tile: reload it (never used)
      tnext = decode(lnext);
      patch_addr(tnext);
      wnext = weight_addr(tnext);
    }
    chunk_body(cc, last, par);
    if (!last) { ++cc; return false; }
    wrow = wnext;
    epilogue(par);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    cc = 0;
    li += wgs;
    tcur = tnext;
    return li >= ntl;
  };
  for (;;) {
    if (advance(std::integral_constant<int, 0>{})) break;
    if (advance(std::integral_constant<int, 1>{})) break;
  }
}

template <typename T, int MODE, int PWID, int BN, bool PART = false>
static int launch_conv3x3_pw(const ConvArgs& a, hipStream_t st) {
  static bool raised = false;
  if (!raised) {
    hipError_t e = hipFuncSetAttribute((const void*)conv3x3_kernel<T, MODE, PWID, BN, PART>, hipFuncAttributeMaxDynamicSharedMemorySize, v2_lds_total(BN));
    if (e != hipSuccess) return (int)e;
    raised = true;
  }
  hipLaunchKernelGGL((conv3x3_kernel<T, MODE, PWID, BN, PART>), dim3(a.grid), dim3(V2_NT), v2_lds_total(BN), st, a);
  return (int)hipGetLastError();
}

template <typename T, int MODE, int BN>
static int launch_conv3x3_inst(const ConvArgs& a, hipStream_t st) {
  if (a.halo_plin) {
    if (a.ksplit >= 1) return (int)hipErrorInvalidValue;
    if constexpr (MODE == M_FLAT) {
      const int pw = a.tw + 2;
      if (a.th * pw > V2_BM || (a.th + 2) * pw + 2 > V2_PPMAX) return (int)hipErrorInvalidValue;
      return launch_conv3x3_pw<T, MODE, 0, BN>(a, st);
    } else {
      return (int)hipErrorInvalidValue;
    }
  }
  if (a.ksplit >= 1) {   // reduction split across workgroups: pixel-major chains in the plain form
    if constexpr (MODE == M_FLAT) {
      if (a.tw + 2 <= kHaloPitchTiny && (a.th + 2) * kHaloPitchTiny <= V2_PPMAX) return launch_conv3x3_pw<T, MODE, kHaloPitchTiny, BN, true>(a, st);
      if (a.tw + 2 <= kHaloPitchNarrow && (a.th + 2) * kHaloPitchNarrow <= V2_PPMAX) return launch_conv3x3_pw<T, MODE, kHaloPitchNarrow, BN, true>(a, st);
      if (a.tw + 2 <= kHaloPitchWide && (a.th + 2) * kHaloPitchWide <= V2_PPMAX) return launch_conv3x3_pw<T, MODE, kHaloPitchWide, BN, true>(a, st);
    }
    return (int)hipErrorInvalidValue;
  }
  if (a.tw + 2 <= kHaloPitchTiny && (a.th + 2) * kHaloPitchTiny <= V2_PPMAX) return launch_conv3x3_pw<T, MODE, kHaloPitchTiny, BN>(a, st);
  if (a.tw + 2 <= kHaloPitchNarrow && (a.th + 2) * kHaloPitchNarrow <= V2_PPMAX) return launch_conv3x3_pw<T, MODE, kHaloPitchNarrow, BN>(a, st);
  if (a.tw + 2 <= kHaloPitchWide && (a.th + 2) * kHaloPitchWide <= V2_PPMAX) return launch_conv3x3_pw<T, MODE, kHaloPitchWide, BN>(a, st);
  return (int)hipErrorInvalidValue;
}

template <typename T>
static int launch_conv3x3_t(const ConvArgs& a, hipStream_t st) {
  // the host checks the preconditions again: a wrong shape here would index outside the patch buffers
  if (a.R != 3 || a.S != 3 || a.stride != 1 || a.pad != 1 || !a.kchunk || a.C % Tr<T>::BKE != 0 || a.C < Tr<T>::BKE || a.th < 1 || a.tw < 1 ||
      a.th * a.tw > V2_BM || a.tiles_m != a.tiles_y * a.tiles_x || (a.halo_bn != 64 && a.halo_bn != 128) ||
      a.tiles_n != (a.K + a.halo_bn - 1) / a.halo_bn || a.dw_w || (a.ksplit < 1 && (!a.vec_out || (a.has_res && !a.vec_res))) ||
      (long long)a.N * a.in_sN >= (1ll << 31) || a.in_sN < 0 || a.in_sH < 0 || a.in_sW < 0 ||
      (a.mode == M_ZIGZAG && (((a.th | a.tw | a.H | a.W) & 1) || a.has_res)))
    return (int)hipErrorInvalidValue;
  if (a.ksplit >= 1) {
    // reduction split: whole shares of channel chunks, raw fp32 sums to part[share][pixel][part_ld]; the kernel takes the
    // pixel's offset in the partial buffer from the output strides
    const int nch = a.C / Tr<T>::BKE;
    if (a.mode != M_FLAT || a.has_res || a.halo_plin || !a.part || ((uintptr_t)a.part & 15) || a.steps_per_split < 1 || a.steps_per_split * a.ksplit != nch ||
        a.part_ld != a.tiles_n * a.halo_bn || a.out_sP != a.part_ld || a.out_sN != (long long)a.OH * a.OW * a.part_ld || a.M_total != a.N * a.OH * a.OW ||
        a.OH != a.H || a.OW != a.W)
      return (int)hipErrorInvalidValue;
  }
  if (a.mode == M_FLAT) return a.halo_bn == 128 ? launch_conv3x3_inst<T, M_FLAT, 128>(a, st) : launch_conv3x3_inst<T, M_FLAT, 64>(a, st);
  if (a.mode == M_ZIGZAG) return a.halo_bn == 128 ? launch_conv3x3_inst<T, M_ZIGZAG, 128>(a, st) : launch_conv3x3_inst<T, M_ZIGZAG, 64>(a, st);
  return (int)hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------------
// Two linked 3x3 / stride 1 / pad 1 convolution chains (Table 1, ConvX -> ConvY; Section 4.1): the first layer
// (at most 4 input channels, read from the caller's fp32 NCHW tensor) -> 64 channels -> 64 channels [-> 2x2 pooling].
// The intermediate tensor is never written to memory: a workgroup owns a TH x TW block of output pixels (at most 128),
// computes the (TH+2) x (TW+2) block of the intermediate that those pixels read (halo recomputed per tile, the paper's
// halo replication) straight into the LDS patch of the second convolution, and runs the second convolution out of it.
// bf16 operands, fp32 accumulation; the intermediate is rounded to bf16 exactly as it would be when stored between two
// separate chains.
//
// Both weight tensors stay in REGISTERS for all tiles of the (persistent) workgroup: a wavefront owns 32 of the 64 output
// channels (4 wavefronts = 2 pixel halves x 2 channel halves), so its B operands of the second convolution are 36
// fragments (9 taps x 4 k-groups) and of the first 3.  The second convolution therefore reads only pixel fragments from
// LDS (one read per MFMA, no barrier between its nine taps), and LDS holds little more than the patch: two workgroups
// share a compute unit, and while one runs the MFMA-bound second convolution the other runs the VALU-bound phases
// (first convolution's epilogue, the chain's epilogue, the import of the next input block).
//
// Phases per tile (barriers between them): P1 first convolution as a transposed MFMA GEMM over the patch positions
// (reduction slot = tap * 4 + channel, 48 slots), scale / shift / ReLU, positions outside the image forced to zero (they
// are the padding of the second convolution); P2 second convolution, 64 pixels x 32 channels per wavefront; then the
// epilogue of the halo kernel (scale / shift / ReLU, zig-zag pooling over lane quads, staging, 16-byte stores).  The
// fp32 input block of the next tile is fetched during P2.
// ---------------------------------------------------------------------------------------------
constexpr int PR_NW = 4, PR_NT = 64 * PR_NW;
constexpr int PR_BM = kPairRows;              // GEMM rows (output pixels) of a tile
constexpr int PR_PPMAX = kPairPatchMax;       // patch positions, (TH+2) x 18
constexpr int PR_PW = kHaloPitchNarrow;       // patch row pitch in pixels
constexpr int PR_C = kPairChannels;           // channels of the intermediate and of the output
constexpr int PR_K1 = kPairRed;               // reduction slots of the first convolution (3 MFMA steps of 16)
constexpr int PR_INMAX = kPairInMax;          // positions of the staged input block, (TH+4) x (TW+4)
constexpr int PR_PBYTES = PR_PPMAX * LDS_ROW;
constexpr int PR_OFF_XIN = PR_PBYTES;
constexpr int PR_OFF_AFF = PR_OFF_XIN + PR_INMAX * 8;
constexpr int PR_OFF_ROWPOS = PR_OFF_AFF + 4 * PR_C * 4;
constexpr int PR_OFF_ROWOFF = PR_OFF_ROWPOS + PR_BM * 4;
constexpr int PR_SPW = 32 * 2 + 8;              // staging row pitch: a wavefront's 32 channels + 8 bytes (18 dwords: the 32 rows of a store pass hit 32 bank pairs)
constexpr int PR_OFF_STAGE = PR_OFF_ROWOFF + PR_BM * 8;   // per wavefront 64 rows (pixels; 16 pooling windows when pooled)
constexpr int PR_LDS = PR_OFF_STAGE + PR_NW * 64 * PR_SPW;

template <int MODE, bool PMAX>
__global__ __launch_bounds__(PR_NT, 2) void conv_pair_kernel(const ConvArgs a) {
  constexpr int BM = PR_BM, NTH = PR_NT, CE = 8;
  constexpr int ROWS = MODE == M_FLAT ? BM : BM / 4;               // staged rows: pixels, or pooled windows
  constexpr int NI = (PR_INMAX * 4 + NTH - 1) / NTH;               // input elements per thread
  static_assert(MODE == M_FLAT || MODE == M_ZIGZAG, "row enumerations of the pair kernel");
  static_assert(PR_OFF_ROWOFF % 8 == 0 && PR_OFF_AFF % 16 == 0 && PR_OFF_STAGE % 8 == 0, "alignment of the tables");

  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char* s_patch = smem;
  unsigned char* s_xin = smem + PR_OFF_XIN;
  float* s_aff = (float*)(smem + PR_OFF_AFF);                     // scale1, shift1, scale2, shift2
  int* s_rowpos = (int*)(smem + PR_OFF_ROWPOS);
  long long* s_rowoff = (long long*)(smem + PR_OFF_ROWOFF);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  unsigned char* wstg = smem + PR_OFF_STAGE + wave * (64 * PR_SPW);   // this wavefront's staging slice
  const int wave_n = wave & 1, wave_m = wave >> 1;
  const int l31 = lane & 31, lhalf = lane >> 5;
  const int lq = l31 >> 2;
  const int lp = (((0x96 >> lq) & 1) << 4) | ((lq >> 1) << 2) | (l31 & 3);   // pixel of a 32-row block held by this lane (as in the halo kernel)
  const int Hp = a.H + 2, IW = a.tw + 4, npix = (a.th + 4) * IW, PP = (a.th + 2) * PR_PW;
  const int nin = a.pair_C * npix;

  // ---- this workgroup's tiles: each XCD owns a contiguous, balanced range (neighbouring tiles share input rows) ----
  const int G = gridDim.x, nx = G < NUM_XCD ? G : NUM_XCD;
  const int xcd = blockIdx.x % nx, wgs = (G - xcd + nx - 1) / nx;
  const int m0 = xcd * a.tiles_m / nx, mlen = (xcd + 1) * a.tiles_m / nx - m0;
  int li = blockIdx.x / nx;
  if (li >= mlen) return;                                          // uniform per workgroup
  // ---- resident weights: this wavefront's 32 channels -------------------------------------------------------------
  u32x4_t w2[36], w1[3];
  {
    const unsigned char* wp = (const unsigned char*)a.w + ((long long)(wave_n * 32 + l31) * a.Kred_pad + lhalf * 8) * 2;
#pragma unroll
    for (int s = 0; s < 36; ++s) w2[s] = *(const u32x4_t*)(wp + ((s >> 2) * PR_C + (s & 3) * 16) * 2);
    const unsigned char* w1p = (const unsigned char*)a.dw_w + ((wave_n * 32 + l31) * PR_K1 + lhalf * 8) * 2;
#pragma unroll
    for (int j = 0; j < 3; ++j) w1[j] = *(const u32x4_t*)(w1p + j * 32);
  }

  // ---- the fp32 input block of a tile: element e = (channel, block row, block column), the same for every tile ------
  // Per element only what does not depend on the tile is kept: its offset from the block's first element in the caller's
  // tensor and its position in the block.  A tile's rows lie in at most two images of the stack (TH + 4 <= H + 2, checked
  // by the host); rows of the second image are `xdelta` elements further than the stacked row count says.
  int xe[NI], xg[NI];                                              // channel << 24 | block row << 12 | block column (-1 = none); offset
#pragma unroll
  for (int it = 0; it < NI; ++it) {
    const int e = tid + it * NTH;
    const int c = e / npix, rem = e - c * npix, ir = rem / IW, ic = rem - ir * IW;
    xe[it] = e < nin ? (c << 24) | (ir << 12) | ic : -1;
    xg[it] = (int)(c * a.pair_sC + ir * a.pair_sH + ic);
  }
  const int xdelta = (int)(a.pair_sN - (long long)Hp * a.pair_sH);
  float xr[NI];
  // image and input row of a stacked row `sr` of a tile whose first row lies in image n0
  auto split_row = [&](int sr, int n0, int& n, int& ih) __attribute__((always_inline)) {
    const int rel = sr - n0 * Hp;
    const bool next = rel >= Hp;
    n = n0 + (next ? 1 : 0);
    ih = rel - (next ? Hp : 0) - 1;
  };
  auto load_xin = [&](int l) __attribute__((always_inline)) {
    const int tile_m = m0 + l, tyi = tile_m / a.tiles_x;
    const int q0 = tyi * a.th, x0 = (tile_m - tyi * a.tiles_x) * a.tw;
    const int n0 = q0 > 0 ? (q0 - 1) / Hp : 0;
    const int rel0 = q0 - 1 - n0 * Hp;                             // block row 0 relative to image n0's first stacked row (-1 at the very top)
    // element offset of block position (0, 0) of channel 0 (may point before the tensor: only valid elements are read)
    const long long base = (long long)n0 * a.pair_sN + (long long)(rel0 - 1) * a.pair_sH + (x0 - 2);
    const float* src = (const float*)a.in + base;
#pragma unroll
    for (int it = 0; it < NI; ++it) {
      const int ir = (xe[it] >> 12) & 0xfff, ic = xe[it] & 0xfff;
      const int rel = rel0 + ir;
      const bool next = rel >= Hp;
      const int ih = rel - (next ? Hp : 0) - 1, n = n0 + (next ? 1 : 0), iw = x0 - 2 + ic;
      const bool ok = xe[it] >= 0 && n < a.N && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
      // (elements outside the images read the tensor's first element instead, so the load needs no branch)
      const float* ptr = ok ? src + (xg[it] + (next ? xdelta : 0)) : (const float*)a.in;
      const float v = *ptr;
      xr[it] = ok ? v : 0.f;
    }
  };
  auto store_xin = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int it = 0; it < NI; ++it) {
      if (xe[it] >= 0) {
        const int c = xe[it] >> 24, ir = (xe[it] >> 12) & 0xfff, ic = xe[it] & 0xfff;
        *(uint16_t*)(s_xin + (ir * IW + ic) * 8 + c * 2) = f2bf(xr[it]);
      }
    }
  };

  // ---- which pixel of the tile a GEMM row is (the conflict-free enumerations of the halo kernel, pitch 18) ----
  auto flat_px = [&](int m, int& ty, int& tx) __attribute__((always_inline)) {
    const int nbx = a.tw >> 1, rows8 = (a.tw & 1) ? 0 : (a.th >> 3) * 8, full = rows8 * a.tw;
    if (m < full) {
      const int b = m >> 4, i = m & 15, by = b / nbx, bx = b - by * nbx;
      ty = by * 8 + (i >> 1); tx = bx * 2 + (i & 1);
    } else {
      const int r = m - full, y = r / a.tw;
      ty = rows8 + y; tx = r - y * a.tw;
    }
  };
  auto zz_win = [&](int w, int& wy, int& wx) __attribute__((always_inline)) {
    const int hw = a.tw >> 1, rows4 = (a.th >> 3) * 4, full = rows4 * hw;
    if (w < full) {
      const int g = w / (4 * hw), r = w - g * 4 * hw;
      wx = r >> 2; wy = g * 4 + (r & 3);
    } else {
      const int r = w - full, y = r / hw;
      wy = rows4 + y; wx = r - y * hw;
    }
  };

  // ---- set-up: scale / shift, row table, zeroed input block ---------------------------------------------------
  for (int i = tid; i < PR_INMAX * 2; i += NTH) ((uint32_t*)s_xin)[i] = 0u;   // channel slots beyond pair_C stay zero
  {
    const int w = tid / PR_C, c = tid - w * PR_C;                  // NTH == 4 * PR_C
    static_assert(NTH == 4 * PR_C, "one thread per folded scale / shift value");
    s_aff[tid] = w == 0 ? a.dw_scale[c] : w == 1 ? a.dw_shift[c] : w == 2 ? a.scale[c] : a.shift[c];
  }
  for (int q = tid; q < ROWS; q += NTH) {
    int y, x;
    if (MODE == M_FLAT) flat_px(q, y, x); else zz_win(q, y, x);
    const bool ok = MODE == M_FLAT ? (y < a.th && x < a.tw) : (2 * y < a.th && 2 * x < a.tw);
    s_rowpos[q] = ok ? (y << 16) | x : -1;
  }
  __syncthreads();
  load_xin(li);
  store_xin();

  // ---- per-lane constants -------------------------------------------------------------------------------------
  // P1: the two taps (4 slots each) this half-wavefront feeds to MFMA step j are taps 4j + 2*lhalf and the next one;
  // taps 9..11 do not exist (zero operand)
  auto tap_off = [&](int j, int h) __attribute__((always_inline)) -> int {
    const int t = 4 * j + 2 * lhalf + h;
    return t < 9 ? ((t / 3) * IW + t % 3) * 8 : -1;
  };
  // P2: this lane's two pixels
  int abase[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int m = wave_m * 64 + i * 32 + lp;
    int ty, tx;
    if (MODE == M_FLAT) flat_px(m, ty, tx);
    else {
      int wy, wx;
      zz_win(m >> 2, wy, wx);
      ty = 2 * wy + ((m >> 1) & 1); tx = 2 * wx + (m & 1);
    }
    abase[i] = ((ty < a.th && tx < a.tw) ? ty * PR_PW + tx : 0) * LDS_ROW + lhalf * 16;
  }
  const int nunits = (PP + 31) / 32;
  const float lo1 = a.dw_relu ? 0.f : -3.4028235e38f, lo2 = a.relu ? 0.f : -3.4028235e38f;
  __syncthreads();

  for (;;) {
    const int tile_m = m0 + li, tyi = tile_m / a.tiles_x;
    const int q0 = tyi * a.th, x0 = (tile_m - tyi * a.tiles_x) * a.tw;
    const int n0 = q0 / Hp;                                        // image of the tile's first output row
    // the next tile's input block is fetched now (first-touch reads from device memory: their latency is covered by
    // both convolutions of this tile) and written to LDS after the second convolution
    const bool more = li + wgs < mlen;
    if (more) load_xin(li + wgs);

    // ---- P1: this wavefront's 32 channels of the intermediate at the patch positions p = 32 * unit + lane % 32 -------
    for (int u = wave_m; u < nunits; u += PR_NW / 2) {
      const int p = u * 32 + l31, pcl = p < PP ? p : PP - 1;
      const int pr = pcl / PR_PW, pc = pcl - pr * PR_PW;
      const unsigned char* xb = s_xin + (pr * IW + pc) * 8;
      f32x16_t c1;
#pragma unroll
      for (int e = 0; e < 16; ++e) c1[e] = 0.f;
#pragma unroll
      for (int j = 0; j < 3; ++j) {
        // (taps beyond the ninth read position 0 of the window: their weight slots are zero and the block holds finite values)
        const int o0 = tap_off(j, 0), o1 = tap_off(j, 1);
        const uint2 t0 = *(const uint2*)(xb + (o0 >= 0 ? o0 : 0));
        const uint2 t1 = *(const uint2*)(xb + (o1 >= 0 ? o1 : 0));
        const u32x4_t fa = {t0.x, t0.y, t1.x, t1.y};
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, w1[j]), __builtin_bit_cast(bf16x8_t, fa), c1, 0, 0, 0);
      }
      int n, ih;
      split_row(q0 + pr, n0, n, ih);
      const int iw = x0 - 1 + pc;
      const bool inside = n < a.N && (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
      if (p < PP) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int c = wave_n * 32 + g * 8 + lhalf * 4;
          const f32x4_t sc = *(const f32x4_t*)(s_aff + c), sh = *(const f32x4_t*)(s_aff + PR_C + c);
          float y[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] = fmx(c1[4 * g + e] * sc[e] + sh[e], lo1);
          uint2 o;
          o.x = inside ? f2bf2(y[0], y[1]) : 0u;                   // positions outside the image: padding of the second convolution
          o.y = inside ? f2bf2(y[2], y[3]) : 0u;
          *(uint2*)(s_patch + p * LDS_ROW + c * 2) = o;
        }
      }
    }
    __syncthreads();

    // (after a barrier that every wavefront reaches only when it has finished the previous tile's epilogue, which has
    // no barrier of its own; published by the barrier after P2)
    // where each staged row goes in the output (element offset of its channel 0; -1 = not an output of this tile)
    for (int q = tid; q < ROWS; q += NTH) {
      const int pos = s_rowpos[q];
      long long ob = -1;
      if (pos >= 0) {
        const int y = pos >> 16, x = pos & 0xffff;
        int n, oh;
        split_row(q0 + (MODE == M_FLAT ? y : 2 * y), n0, n, oh);
        oh += 1;                                                   // (split_row returns the input row of a patch position)
        const int ow = x0 + (MODE == M_FLAT ? x : 2 * x);
        if (n < a.N && oh < a.H && ow < a.W)
          ob = (long long)n * a.out_sN + (MODE == M_FLAT ? (long long)(oh * a.OW + ow) : (long long)((oh >> 1) * a.PW + (ow >> 1))) * a.out_sP;
      }
      s_rowoff[q] = ob;
    }

    // ---- P2: the second convolution out of the patch ------------------------------------------------------------
    f32x16_t acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    {
      constexpr int NS = 36, DEPTH = 1;                            // (tap, k-group) steps; fragments fetched DEPTH steps ahead
      u32x4_t fa[DEPTH + 1][2];
      auto fetch = [&](int s, int slot) __attribute__((always_inline)) {
        const int tap = s >> 2, kg = s & 3;
#pragma unroll
        for (int i = 0; i < 2; ++i) fa[slot][i] = *(const u32x4_t*)(s_patch + abase[i] + ((tap / 3) * PR_PW + tap % 3) * LDS_ROW + kg * 32);
      };
#pragma unroll
      for (int s = 0; s < DEPTH; ++s) fetch(s, s);
#pragma unroll
      for (int s = 0; s < NS; ++s) {
        if (s + DEPTH < NS) fetch(s + DEPTH, (s + DEPTH) % (DEPTH + 1));
#pragma unroll
        for (int i = 0; i < 2; ++i)
          acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, w2[s]),
                                                           __builtin_bit_cast(bf16x8_t, fa[s % (DEPTH + 1)][i]), acc[i], 0, 0, 0);
      }
    }
    if (more) store_xin();
    __syncthreads();                                               // the patch is free: the next tile's P1 may write it

    // ---- epilogue: scale / shift / ReLU, pooling over the lane quad; every wavefront stages its own 64 pixels x 32
    // channels in the output type in a private LDS slice (LDS serves a wavefront's requests in order) and stores them as
    // whole 16-byte channel groups: no barrier
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int srow = MODE == M_FLAT ? i * 32 + lp : ((i * 32 + lp) >> 2);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int cl = g * 8 + lhalf * 4, c = wave_n * 32 + cl;
        const f32x4_t sc = *(const f32x4_t*)(s_aff + 2 * PR_C + c), sh = *(const f32x4_t*)(s_aff + 3 * PR_C + c);
        float y[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = fmx(acc[i][4 * g + e] * sc[e] + sh[e], lo2);
        bool mine = true;
        if (MODE == M_ZIGZAG) {
          // the window's four pixels are lanes 4w .. 4w+3: butterfly over the quad, lane i keeps group g == i
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            y[e] = PMAX ? quad_max<true>(y[e]) : quad_add<true>(y[e]);
            y[e] = PMAX ? quad_max<false>(y[e]) : quad_add<false>(y[e]) * 0.25f;
          }
          mine = (l31 & 3) == g;
        }
        if (mine) {
          uint2 o;
          o.x = f2bf2(y[0], y[1]);
          o.y = f2bf2(y[2], y[3]);
          *(uint2*)(wstg + srow * PR_SPW + cl * 2) = o;
        }
      }
    }
    {
      constexpr int PROWS = MODE == M_FLAT ? 64 : 16, G = 4, NGW = PROWS * G / 64;   // 16-byte groups of the slice per lane
      const int qbase = MODE == M_FLAT ? wave_m * 64 : wave_m * 16;
      long long ob[NGW];
      u32x4_t v[NGW];
#pragma unroll
      for (int u = 0; u < NGW; ++u) {
        const int idx = lane + u * 64, r = idx / G, cg = idx % G;
        ob[u] = s_rowoff[qbase + r];
        const uint2 lo8 = *(const uint2*)(wstg + r * PR_SPW + cg * 16), hi8 = *(const uint2*)(wstg + r * PR_SPW + cg * 16 + 8);
        v[u] = u32x4_t{lo8.x, lo8.y, hi8.x, hi8.y};
      }
#pragma unroll
      for (int u = 0; u < NGW; ++u) {
        const int cg = (lane + u * 64) % G;
        if (ob[u] >= 0) *(u32x4_t*)((bf16_t*)a.out + ob[u] + wave_n * 32 + cg * CE) = v[u];
      }
    }
    li += wgs;
    if (li >= mlen) break;
  }
}

static int launch_pair(const ConvArgs& a, int dtype, hipStream_t st) {
  // the host checks every shape the kernel's LDS layout and indexing assume
  if (dtype != DT_BF16 || !a.pair || a.pair_C < 1 || a.pair_C > 4 || a.C != PR_C || a.K != PR_C || a.R != 3 || a.S != 3 || a.stride != 1 ||
      a.pad != 1 || !a.kchunk || a.Kred_pad != 9 * PR_C || !a.dw_w || !a.dw_scale || !a.dw_shift || !a.vec_out || a.out_f32 || a.has_res ||
      a.ksplit >= 1 || a.th < 1 || a.tw < 1 || a.th * a.tw > PR_BM || a.tw + 2 > PR_PW || (a.th + 2) * PR_PW > PR_PPMAX ||
      (a.th + 4) * (a.tw + 4) > PR_INMAX || (a.th + 3) * (a.tw + 4) + 20 > PR_INMAX || a.th + 4 >= 4096 || a.tw + 4 >= 4096 || a.tiles_x != (a.W + a.tw - 1) / a.tw ||
      (long long)a.tiles_y * a.th < (long long)a.N * (a.H + 2) || a.tiles_m != a.tiles_y * a.tiles_x || a.tiles_n != 1 ||
      (long long)a.N * (a.H + 2) + a.th + 4 >= (1ll << 31) || a.OH != a.H || a.OW != a.W || a.th + 4 > a.H + 2 ||
      (long long)a.N * a.pair_sN + (long long)4 * a.pair_sC >= (1ll << 31) || a.pair_sN < 0 || a.pair_sC < 0 || a.pair_sH < 0 ||
      (a.mode == M_ZIGZAG && (((a.th | a.tw | a.H | a.W) & 1) || (a.pool != POOL_MAX && a.pool != POOL_AVG) || 2 * a.PH != a.H || 2 * a.PW != a.W)) ||
      (a.mode == M_FLAT && a.pool != POOL_NONE) || (a.mode != M_FLAT && a.mode != M_ZIGZAG))
    return (int)hipErrorInvalidValue;
  if (a.mode == M_FLAT) hipLaunchKernelGGL((conv_pair_kernel<M_FLAT, false>), dim3(a.grid), dim3(PR_NT), PR_LDS, st, a);
  else if (a.pool == POOL_MAX) hipLaunchKernelGGL((conv_pair_kernel<M_ZIGZAG, true>), dim3(a.grid), dim3(PR_NT), PR_LDS, st, a);
  else hipLaunchKernelGGL((conv_pair_kernel<M_ZIGZAG, false>), dim3(a.grid), dim3(PR_NT), PR_LDS, st, a);
  return (int)hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Fully connected chain with few rows (a batch of at most 32 images; Table 4, FullyConnected): out[m][k] = sum_i x[m][i] *
// w[k][i].  Every weight is used once per image, so the chain is bound by streaming the weights from device memory and
// what matters is how many bytes are in flight and that memory is read in long sequential runs: a wavefront owns 32
// output channels and a share of the reduction, its weight fragments are packed in the order it loads them (every
// load instruction reads 1 KB of consecutive memory, a share is one sequential stream) and go straight from memory
// into the registers the MFMA reads them from, FC_DEPTH steps of 64 reduction elements ahead (16 KB in flight per
// wavefront), with no LDS and no barrier anywhere; the activation fragments (a few MB, cache resident) travel the same way.  The operator split is output channels first, then the
// reduction (Section 4.2.2: a C / R / S split needs an additional reduction): the shares are raw fp32 sums in
// part[z][m][k], added in index order by the summing pass, which also applies the chain's epilogue.
// bf16 operands, fp32 accumulation.  Rows m >= M read row 0 and are not stored.
// ---------------------------------------------------------------------------------------------
constexpr int FC_NW = 4, FC_NT = 64 * FC_NW, FC_BN = 32 * FC_NW, FC_DEPTH = 4;

__global__ __launch_bounds__(FC_NT, 2) void fc_stream_kernel(const ConvArgs a) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, lhalf = lane >> 5;
  // Reduction shared out across workgroups (a.ksplit >= 1: a workgroup owns 128 channels, a wavefront 32 of them, and share z
  // of the steps; raw sums go to the summing pass), or, for a short reduction (a.ksplit < 1), across the four wavefronts of
  // a workgroup that owns 32 channels: every wavefront then has all its steps in flight at once (one memory round trip
  // instead of one per FC_DEPTH steps), the four partial sums meet in LDS and the chain's epilogue runs here.
  const bool direct = a.ksplit < 1;
  const int tile_n = direct ? 0 : blockIdx.x % a.tiles_n, z = direct ? wave : blockIdx.x / a.tiles_n;
  const int nsteps_all = a.Kred_pad / 64;
  const int sps = direct ? (nsteps_all + FC_NW - 1) / FC_NW : a.steps_per_split;
  const int s0 = z * sps;
  const int ns = nsteps_all - s0 < sps ? nsteps_all - s0 : sps;
  if (ns <= 0 && !direct) return;                                  // (uniform per workgroup)
  const int k0 = direct ? (int)blockIdx.x * 32 : tile_n * FC_BN + wave * 32;   // first output channel of this wavefront
  // weights: [32-channel block][step][k-group][lane][8 elements], the order in which this wavefront loads them
  const unsigned char* wp = (const unsigned char*)a.w + ((((long long)(k0 / 32) * nsteps_all + s0) * 4 * 64 + lane) * 16);
  // activations: row m of the flattened input (reduction index = position in the NHWC tensor of an image)
  const int m = l31 < a.M_total ? l31 : 0;
  const unsigned char* xp = (const unsigned char*)a.in + (((long long)m * a.in_sN + (long long)s0 * 64 + lhalf * 8) * 2);

  u32x4_t fw[FC_DEPTH][4], fx[FC_DEPTH][4];
  auto fetch = [&](int slot, int step) __attribute__((always_inline)) {
    const int sc = step < ns ? step : ns - 1;                      // beyond the share: re-read its last step (never used)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      fw[slot][g] = *(const u32x4_t*)(wp + (sc * 4 + g) * 1024);
      fx[slot][g] = *(const u32x4_t*)(xp + sc * 128 + g * 32);
    }
  };
  f32x16_t acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  if (ns > 0) {                                                    // (a wavefront of the direct form may have no step)
#pragma unroll
    for (int d = 0; d < FC_DEPTH; ++d) fetch(d, d);
  }
  for (int s = 0; s < ns; s += FC_DEPTH) {
#pragma unroll
    for (int d = 0; d < FC_DEPTH; ++d) {
      if (s + d < ns) {
#pragma unroll
        for (int g = 0; g < 4; ++g)
          acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fw[d][g]), __builtin_bit_cast(bf16x8_t, fx[d][g]), acc, 0, 0, 0);
      }
      fetch(d, s + d + FC_DEPTH);
    }
  }
  // accumulator rows = channels, columns = images: this lane holds 4 groups of 4 consecutive channels of image l31
  if (direct) {
    // the four wavefronts' sums of the same 32 channels x 32 images, added in wavefront order; wavefront w finishes
    // accumulator elements 4w .. 4w + 3 of every lane
    __shared__ float s_red[FC_NW][16][64];
#pragma unroll
    for (int e = 0; e < 16; ++e) s_red[wave][e][lane] = acc[e];
    __syncthreads();
    if (l31 < a.M_total) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int e = wave * 4 + q;
        float sum = s_red[0][e][lane];
#pragma unroll
        for (int w = 1; w < FC_NW; ++w) sum += s_red[w][e][lane];
        const int k = k0 + (e >> 2) * 8 + lhalf * 4 + (e & 3);
        if (k < a.K) {
          float v = sum * a.scale[k] + a.shift[k];
          if (a.relu) v = fmx(v, 0.f);
          const long long o = (long long)l31 * a.out_sN + (long long)k * a.out_sK;
          if (a.out_f32) ((float*)a.out)[o] = v; else ((uint16_t*)a.out)[o] = f2bf(v);
        }
      }
    }
    return;
  }
  if (l31 < a.M_total) {
    float* dst = a.part + ((long long)z * a.M_total + l31) * a.part_ld + k0;
#pragma unroll
    for (int g = 0; g < 4; ++g)
      *(f32x4_t*)(dst + g * 8 + lhalf * 4) = f32x4_t{acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
  }
}

static int launch_fc(const ConvArgs& a, int dtype, hipStream_t st) {
  // the host checks what the kernel's indexing assumes
  if (dtype != DT_BF16 || a.mode != M_FLAT || a.OH != 1 || a.OW != 1 || a.R != a.H || a.S != a.W || a.pad != 0 || a.M_total < 1 || a.M_total > 32 ||
      a.M_total != a.N || a.kchunk || a.Kred != a.R * a.S * a.C || a.Kred_pad != a.Kred || a.Kred % 64 != 0 || a.in_f32 || a.dw_w || a.pair ||
      (a.H * a.W > 1 && (a.in_sW != a.C || a.in_sH != (long long)a.W * a.C)) || a.in_sN < a.Kred || a.in_sN % 8 != 0 || ((uintptr_t)a.in & 15) != 0 ||
      a.steps_per_split < 1 || a.tiles_n != (a.K + FC_BN - 1) / FC_BN ||
      (a.ksplit >= 1 && ((long long)a.ksplit * a.steps_per_split < a.Kred_pad / 64 || !a.part || a.part_ld < a.tiles_n * FC_BN || a.part_ld % 4 != 0 ||
                         ((uintptr_t)a.part & 15) != 0 || a.grid != a.tiles_n * a.ksplit)) ||
      (a.ksplit < 1 && (a.steps_per_split < a.Kred_pad / 64 || a.grid != (a.K + 31) / 32 || a.has_res || !a.out || !a.scale || !a.shift)))
    return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(fc_stream_kernel, dim3(a.grid), dim3(FC_NT), 0, st, a);
  return (int)hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// First-layer chain: a dense convolution with a short reduction C*R*S <= 160 (the 3-channel image layer: 3x3 -> 27,
// 7x7 -> 147), reading the caller's graph input where it lies (any strides, fp32 or the compute type) and writing
// the consumer's NHWC layout: the layout transform at the graph boundary (transpose operator, Table 3) is linked
// into its consumer (Section 4.1), so the input is read once and no converted copy is written.
//
// The GEMM is computed transposed (rows = output channels, columns = pixels): in the MFMA accumulator layout a
// lane then owns 4 consecutive channels of one pixel, which it scales, shifts and clamps in registers.
// One wavefront = 32 consecutive output pixels x all K = 32*KB channels; the reduction runs in passes of 32: in
// pass p lane (pixel, h) holds the slots k(i) = 32*p + (i/8)*16 + h*8 + i%8, i = 0..15 (bf16: two 8-element MFMA
// operands; fp32: 16 single ones), gathered through the table `ktab` = {input offset, tap row / column} per slot.
// ---------------------------------------------------------------------------------------------
template <typename T, int KB>
__global__ __launch_bounds__(NT, sizeof(T) == 2 ? 4 : 2) void stem_kernel(const ConvArgs a) {
  using tr = Tr<T>;
  __shared__ __align__(16) float s_scale[KB * 32];
  __shared__ __align__(16) float s_shift[KB * 32];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l31 = lane & 31, h = lane >> 5;
  constexpr int CPP = KB * 32 * (int)sizeof(T) / 16;                 // 16-byte chunks per output pixel
  constexpr int PPI = 64 / CPP;                                      // pixels per store instruction
  constexpr int SPITCH = KB * 32 * (int)sizeof(T) + 16;              // staging row pitch (odd number of 16-byte slots)
  __shared__ __align__(16) unsigned char s_stage[(NT / 64) * 32 * SPITCH];
  __shared__ int2 s_tab[kStemPasses][2][16];                        // per pass, lane half and slot: {input offset, (r << 16) | s}
  const int npass = (a.Kred + 31) / 32;                             // 32-deep MFMA passes over the reduction (<= kStemPasses)
  if (tid < KB * 32) { s_scale[tid] = a.scale[tid]; s_shift[tid] = a.shift[tid]; }
  if (tid < npass * 32) {
    const int p = tid >> 5, hh = (tid >> 4) & 1, i = tid & 15, k = p * 32 + (i / 8) * 16 + hh * 8 + i % 8;
    s_tab[p][hh][i] = make_int2(a.ktab[2 * k], a.ktab[2 * k + 1]);
  }
  __syncthreads();
  // weight operands of one pass: channel 32*b + l31, the same reduction slots
  constexpr int WV = sizeof(T) == 2 ? 1 : 2;                         // 16-byte vectors per 8 elements
  u32x4_t wn[KB][2][WV];
  auto load_w = [&](int p) {
#pragma unroll
    for (int b = 0; b < KB; ++b)
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int v = 0; v < WV; ++v)
          wn[b][q][v] = *(const u32x4_t*)((const unsigned char*)a.w +
                                          ((size_t)(32 * b + l31) * a.Kred_pad + p * 32 + q * 16 + h * 8) * sizeof(T) + v * 16);
  };

  const int OHW = a.OH * a.OW, nblk = a.tiles_m, bstride = gridDim.x * (NT / 64);
  auto gather = [&](int blk, int pass, float* v) {
    const int m = blk * 32 + l31;
    const bool valid = m < a.M_total;
    const int mm = valid ? m : 0;
    const int n = mm / OHW, p = mm - n * OHW, oy = p / a.OW, ox = p - oy * a.OW;
    const int iy0 = oy * a.stride - a.pad, ix0 = ox * a.stride - a.pad;
    const long long base = (long long)n * a.in_sN + (long long)iy0 * a.in_sH + (long long)ix0 * a.in_sW;
    // blocks whose 32 windows lie inside the image (most of them) skip the per-tap bounds tests
    const bool inside = valid && iy0 >= 0 && ix0 >= 0 && iy0 + a.R <= a.H && ix0 + a.S <= a.W;
    if (__all(inside)) {
      if (a.in_f32) {
        const float* pb = (const float*)a.in + base;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int2 t = s_tab[pass][h][i];
          const float x = pb[(t.y >> 16) < a.R ? t.x : 0];            // padding slots of the reduction read a valid address ...
          v[i] = (t.y >> 16) < a.R ? x : 0.f;                          // ... and contribute zero
        }
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          const int2 t = s_tab[pass][h][i];
          const float x = tr::ld(a.in, base + ((t.y >> 16) < a.R ? t.x : 0));
          v[i] = (t.y >> 16) < a.R ? x : 0.f;
        }
      }
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int2 t = s_tab[pass][h][i];
        const bool ok = valid && (unsigned)(iy0 + (t.y >> 16)) < (unsigned)a.H && (unsigned)(ix0 + (t.y & 0xffff)) < (unsigned)a.W;
        const long long idx = ok ? base + t.x : 0;
        const float x = a.in_f32 ? ((const float*)a.in)[idx] : tr::ld(a.in, idx);
        v[i] = ok ? x : 0.f;
      }
    }
  };

  // Steps = (pixel block, pass) pairs in sequence; the gather (and, with several passes, the weights) of the next
  // step are in flight while the current one is multiplied.
  int blk = blockIdx.x * (NT / 64) + wave, pass = 0;
  float vn[16];
  if (blk < nblk) { gather(blk, 0, vn); load_w(0); }
  f32x16_t acc[KB];
#pragma unroll
  for (int b = 0; b < KB; ++b)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[b][e] = 0.f;
  while (blk < nblk) {
    float v[16];
    u32x4_t wf[KB][2][WV];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = vn[i];
#pragma unroll
    for (int b = 0; b < KB; ++b)
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int w = 0; w < WV; ++w) wf[b][q][w] = wn[b][q][w];
    const int cur_blk = blk;
    const bool last_pass = pass == npass - 1;
    if (last_pass) { blk += bstride; pass = 0; } else ++pass;
    if (blk < nblk) {
      gather(blk, pass, vn);
      if (npass > 1) load_w(pass);
    }
    if constexpr (sizeof(T) == 2) {
      const u32x4_t p0 = tr::pack(v), p1 = tr::pack(v + 8);        // round the image to the compute type
#pragma unroll
      for (int b = 0; b < KB; ++b) {
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, wf[b][0][0]),
                                                         __builtin_bit_cast(bf16x8_t, p0), acc[b], 0, 0, 0);
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, wf[b][1][0]),
                                                         __builtin_bit_cast(bf16x8_t, p1), acc[b], 0, 0, 0);
      }
    } else {
#pragma unroll
      for (int b = 0; b < KB; ++b)
#pragma unroll
        for (int i = 0; i < 16; ++i)
          acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(wf[b][i / 8][(i % 8) / 4][i % 4]), v[i], acc[b], 0, 0, 0);
    }
    if (!last_pass) continue;
    // epilogue: lane = pixel l31, channels 32*b + 8*g + 4*h + (0..3) in accumulator elements 4*g + (0..3).  The
    // finished values are transposed through this wavefront's LDS slice so that every store instruction writes
    // whole pixels (contiguous K*sizeof(T)-byte rows) instead of 4-channel fragments of 32 different pixels.
    unsigned char* stg = s_stage + wave * (32 * SPITCH);
#pragma unroll
    for (int b = 0; b < KB; ++b)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int c0 = 32 * b + 8 * g + 4 * h;
        const f32x4_t sc = *(const f32x4_t*)&s_scale[c0], sh = *(const f32x4_t*)&s_shift[c0];
        float y[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          y[j] = acc[b][4 * g + j] * sc[j] + sh[j];
          if (a.relu) y[j] = fmx(y[j], 0.f);
        }
        if constexpr (sizeof(T) == 2) {
          uint2 o;
          o.x = f2bf2(y[0], y[1]);
          o.y = f2bf2(y[2], y[3]);
          *(uint2*)(stg + l31 * SPITCH + c0 * 2) = o;
        } else {
          *(f32x4_t*)(stg + l31 * SPITCH + c0 * 4) = f32x4_t{y[0], y[1], y[2], y[3]};
        }
      }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < 32 / PPI; ++it) {
      const int px = it * PPI + lane / CPP, ch = lane % CPP;
      const u32x4_t o = *(const u32x4_t*)(stg + px * SPITCH + ch * 16);
      const int m = cur_blk * 32 + px;
      if (m < a.M_total) {
        const int n = m / OHW, p = m - n * OHW;
        *(u32x4_t*)((unsigned char*)a.out + ((long long)n * a.out_sN + (long long)p * a.out_sP) * (long long)sizeof(T) + ch * 16) = o;
      }
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int b = 0; b < KB; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[b][e] = 0.f;
  }
}

template <typename T>
static int launch_stem_t(const ConvArgs& a, hipStream_t st) {
  // what the kernel assumes: one 32-deep pass, K = 32 or 64, pixel-major rows, plain chain, aligned NHWC output
  const int esz = (int)sizeof(T);
  if (a.Kred > kStemRed || a.Kred_pad < (a.Kred + 31) / 32 * 32 || !a.ktab || a.mode != M_FLAT || a.has_res || a.pool != POOL_NONE || a.dw_w || a.ksplit >= 1 ||
      a.out_sK != 1 || (a.out_f32 && esz != 4) || (a.out_sP * esz) % 16 != 0 || (a.out_sN * esz) % 16 != 0 ||
      ((uintptr_t)a.out & 15) || ((uintptr_t)a.w & 15) || (a.Kred_pad * esz) % 16 != 0 || a.H > 8192 ||
      a.tiles_m != (a.M_total + 31) / 32 || a.M_total != a.N * a.OH * a.OW)
    return (int)hipErrorInvalidValue;
  if (a.K == 32) hipLaunchKernelGGL((stem_kernel<T, 1>), dim3(a.grid), dim3(NT), 0, st, a);
  else if (a.K == 64) hipLaunchKernelGGL((stem_kernel<T, 2>), dim3(a.grid), dim3(NT), 0, st, a);
  else return (int)hipErrorInvalidValue;
  return (int)hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// First-layer chain with the input block staged on chip (bf16 path; at most 4 input channels read from the caller's
// fp32 NCHW tensor, square kernel up to 7x7, stride 1 or 2, K = 32 or 64).  stem_kernel gathers every element of every
// window from memory (up to 80 single loads per pixel for a 7x7 kernel: bound by address processing, not by bytes);
// here a workgroup owns a TH x TW block of output pixels of one image, reads the input block those windows cover ONCE
// (coalesced along W), keeps it in LDS as [position][4 channels] bf16, and gathers the MFMA operands from LDS: the
// reduction slot is tap * 4 + channel, so one 8-byte LDS read is one tap of one pixel, two taps per lane and MFMA
// step.  The weights of all steps stay in registers for all tiles of the workgroup.  One wavefront = 32 pixels (two
// tile rows of 16) x all K channels; epilogue and whole-pixel stores as in stem_kernel.
// ---------------------------------------------------------------------------------------------
constexpr int SL_NW = 4, SL_NT = 64 * SL_NW;
constexpr int SL_TH = kStemLdsTh, SL_TW = kStemLdsTw;             // output pixels of a tile: 8 x 16 = 4 wavefronts x 32
constexpr int SL_INMAX = kStemLdsInMax;                            // positions of the staged input block
static_assert(SL_TH * SL_TW == 32 * SL_NW && SL_TW == 16, "one wavefront = two tile rows of 16 pixels");

// positions of the staged input block by kernel size class (NSTEP MFMA steps of four taps): up to 3x3 at stride 2 a block is
// at most 17 x 33 or 15 x 35 positions, up to 5x5 19 x 35; the host checks the launch against these
constexpr int sl_inpos(int nstep) { return nstep <= 3 ? 576 : nstep <= 7 ? 672 : SL_INMAX; }
static_assert(sl_inpos(3) == 576 && sl_inpos(7) == 672, "the same limits as stem_lds_in_positions(), which the host checks");

// (the small kernels keep three or six weight fragments per lane, so four or three workgroups share a compute unit instead of
// two: a tile is a chain of short dependent phases, and what hides their latencies is other tiles in flight.  Measured at
// batch 32 on the 3x3 / 2 first layers with a linked pooling: 64 channels 33.7 -> 30.3 us with three workgroups (30.8 with four,
// which spills), 24 channels padded to 32: 28.3 -> 23.5 us with four)
template <int KB, int NSTEP, bool POOL>
__global__ __launch_bounds__(SL_NT, NSTEP <= 3 ? (KB == 1 ? 4 : 3) : 2) void stem_lds_kernel(const ConvArgs a) {
  constexpr int K = KB * 32;
  constexpr int SPITCH = K * 2 + 16;                               // staging row pitch (odd number of 16-byte slots)
  constexpr int CPP = K * 2 / 16, PPI = 64 / CPP;                  // 16-byte chunks per output pixel, pixels per store instruction
  __shared__ __align__(16) unsigned char s_xin[SL_INMAX * 8];
  __shared__ __align__(16) unsigned char s_stage[SL_NW * 32 * SPITCH];
  __shared__ __align__(16) float s_aff[2 * K];
  __shared__ int2 s_tap[NSTEP][2];                                 // per step and lane half: LDS byte offsets of its two taps (-1 = none)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l31 = lane & 31, lhalf = lane >> 5;
  const int st = a.stride;
  // convolution pixels of a tile: TH x TW, or, with a linked max-pooling, the CH x CW block that the tile's pph x ppw
  // pooling windows cover (window overlap recomputed per tile; at most 128 pixels = one per lane of the 4 wavefronts)
  const int CH = POOL ? (a.pph - 1) * a.ps + a.pk : SL_TH, CW = POOL ? (a.ppw - 1) * a.ps + a.pk : SL_TW;
  const int IH = (CH - 1) * st + a.R, IW = (CW - 1) * st + a.S, npos = IH * IW, nin = a.pair_C * npos;
  const int ntaps = a.R * a.S;

  for (int i = tid; i < SL_INMAX * 2; i += SL_NT) ((uint32_t*)s_xin)[i] = 0u;   // channel slots beyond pair_C stay zero
  if (tid < 2 * K) s_aff[tid] = tid < K ? a.scale[tid] : a.shift[tid - K];
  if (tid < NSTEP * 2) {
    const int j = tid >> 1, hh = tid & 1, t0 = 4 * j + 2 * hh, t1 = t0 + 1;
    s_tap[j][hh] = make_int2(t0 < ntaps ? ((t0 / a.S) * IW + t0 % a.S) * 8 : -1, t1 < ntaps ? ((t1 / a.S) * IW + t1 % a.S) * 8 : -1);
  }
  // resident weights: rows = channels 32 * b + l31, [K][NSTEP * 16] with slot = tap * 4 + channel
  u32x4_t w[NSTEP][KB];
#pragma unroll
  for (int j = 0; j < NSTEP; ++j)
#pragma unroll
    for (int b = 0; b < KB; ++b)
      w[j][b] = *(const u32x4_t*)((const unsigned char*)a.dw_w + ((32 * b + l31) * (NSTEP * 16) + j * 16 + lhalf * 8) * 2);
  // this lane's convolution pixel of the tile and where its window starts in the staged block
  const int q = wave * 32 + l31;
  const bool qok = q < CH * CW;
  const int ty = qok ? q / CW : 0, tx = qok ? q - ty * CW : 0;
  const int xbase = ((ty * st) * IW + tx * st) * 8;
  const float lo = a.relu ? 0.f : -3.4028235e38f;
  unsigned char* stg = s_stage + wave * (32 * SPITCH);
  const int tiles_img = a.tiles_y * a.tiles_x;

  // ---- the input block of a tile: element e = (channel, block row, block column), consecutive threads along W; what does
  // not depend on the tile (position in the block, offset from the block's first element) is worked out once ----------
  constexpr int NI = (sl_inpos(NSTEP) * 4 + SL_NT - 1) / SL_NT;
  int xe[NI], xg[NI];
#pragma unroll
  for (int it = 0; it < NI; ++it) {
    const int e = tid + it * SL_NT;
    const int c = e / npos, rem = e - c * npos, ir = rem / IW, ic = rem - ir * IW;
    xe[it] = e < nin ? (c << 24) | (ir << 12) | ic : -1;
    xg[it] = (int)(c * a.pair_sC + ir * a.pair_sH + ic);
  }
  float xr[NI];
  // first convolution pixel of a tile (may lie outside the map when the pooling is padded)
  auto tile_origin = [&](int tile, int& n, int& cy0, int& cx0) __attribute__((always_inline)) {
    n = tile / tiles_img;
    const int tr = tile - n * tiles_img, tyi = tr / a.tiles_x, txi = tr - tyi * a.tiles_x;
    cy0 = POOL ? tyi * a.pph * a.ps - a.pp : tyi * SL_TH;
    cx0 = POOL ? txi * a.ppw * a.ps - a.pp : txi * SL_TW;
  };
  auto load_block = [&](int tile) __attribute__((always_inline)) {
    int n, cy0, cx0;
    tile_origin(tile, n, cy0, cx0);
    const int iy0 = cy0 * st - a.pad, ix0 = cx0 * st - a.pad;
    // (may point before the tensor: only elements inside the image are read, the others read the tensor's first element)
    const float* src = (const float*)a.in + ((long long)n * a.pair_sN + (long long)iy0 * a.pair_sH + ix0);
#pragma unroll
    for (int it = 0; it < NI; ++it) {
      const int ir = (xe[it] >> 12) & 0xfff, ic = xe[it] & 0xfff;
      const bool ok = xe[it] >= 0 && (unsigned)(iy0 + ir) < (unsigned)a.H && (unsigned)(ix0 + ic) < (unsigned)a.W;
      const float* ptr = ok ? src + xg[it] : (const float*)a.in;
      const float v = *ptr;
      xr[it] = ok ? v : 0.f;
    }
  };
  auto store_block = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int it = 0; it < NI; ++it) {
      if (xe[it] >= 0) {
        const int c = xe[it] >> 24, ir = (xe[it] >> 12) & 0xfff, ic = xe[it] & 0xfff;
        *(uint16_t*)(s_xin + (ir * IW + ic) * 8 + c * 2) = f2bf(xr[it]);
      }
    }
  };

  // pooling stage: the window and 16-byte channel group this thread finishes in the first round
  const int pl_wi = tid / CPP, pl_ch = tid - pl_wi * CPP, pl_wy = POOL ? pl_wi / a.ppw : 0, pl_wx = POOL ? pl_wi - pl_wy * a.ppw : 0;

  int tile = blockIdx.x;
  if (tile < a.tiles_m) load_block(tile);
  while (tile < a.tiles_m) {
    int n, cy0, cx0;
    tile_origin(tile, n, cy0, cx0);
    __syncthreads();                                               // the previous tile's reads of the block and of the staging are done
    store_block();
    __syncthreads();
    const int next = tile + gridDim.x;
    if (next < a.tiles_m) load_block(next);                        // in flight during this tile's convolution and stores
    // ---- the convolution of this wavefront's 32 pixels ----------------------------------------------------------
    f32x16_t acc[KB];
#pragma unroll
    for (int b = 0; b < KB; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[b][e] = 0.f;
#pragma unroll
    for (int j = 0; j < NSTEP; ++j) {
      const int2 t = s_tap[j][lhalf];
      // (slots beyond the last tap read position 0 of the window: their weights are zero and the block holds finite values)
      const uint2 t0 = *(const uint2*)(s_xin + xbase + (t.x >= 0 ? t.x : 0));
      const uint2 t1 = *(const uint2*)(s_xin + xbase + (t.y >= 0 ? t.y : 0));
      const u32x4_t fa = {t0.x, t0.y, t1.x, t1.y};
#pragma unroll
      for (int b = 0; b < KB; ++b)
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, w[j][b]), __builtin_bit_cast(bf16x8_t, fa), acc[b], 0, 0, 0);
    }
    // ---- epilogue: lane = pixel l31, channels 32*b + 8*g + 4*lhalf + (0..3); transposed through this wavefront's LDS
    // slice so that every store instruction writes whole pixels.  With a linked pooling, pixels outside the map are
    // staged as -infinity (padding never wins a maximum) ------------------------------------------------------------
    const bool inmap = !POOL || (qok && (unsigned)(cy0 + ty) < (unsigned)a.OH && (unsigned)(cx0 + tx) < (unsigned)a.OW);
#pragma unroll
    for (int b = 0; b < KB; ++b)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int c0 = 32 * b + 8 * g + 4 * lhalf;
        const f32x4_t sc = *(const f32x4_t*)&s_aff[c0], sh = *(const f32x4_t*)&s_aff[K + c0];
        float y[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = fmx(acc[b][4 * g + e] * sc[e] + sh[e], lo);
        uint2 o;
        o.x = f2bf2(y[0], y[1]);
        o.y = f2bf2(y[2], y[3]);
        if (POOL && !inmap) o = uint2{0xff80ff80u, 0xff80ff80u};
        *(uint2*)(stg + l31 * SPITCH + c0 * 2) = o;
      }
    if constexpr (POOL) {
      // ---- linked max-pooling: one thread = one 16-byte channel group of one pooling window of the tile -------------
      __syncthreads();
      const int tr = tile - n * tiles_img, tyi = tr / a.tiles_x, txi = tr - tyi * a.tiles_x;
      for (int idx = tid; idx < a.pph * a.ppw * CPP; idx += SL_NT) {
        // (the first round's window and channel group are the same for every tile: worked out once, before the tile loop)
        int wi = pl_wi, ch = pl_ch, wy = pl_wy, wx = pl_wx;
        if (idx != tid) { wi = idx / CPP; ch = idx - wi * CPP; wy = wi / a.ppw; wx = wi - wy * a.ppw; }
        const int py = tyi * a.pph + wy, px = txi * a.ppw + wx;
        if (py >= a.PH || px >= a.PW) continue;
        float m[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) m[e] = -INFINITY;
        if (a.pk == 3) {
          // (all nine reads of the window before the first maximum: one LDS latency, not nine)
          u32x4_t wv9[9];
#pragma unroll
          for (int t9 = 0; t9 < 9; ++t9)
            wv9[t9] = *(const u32x4_t*)(s_stage + ((wy * a.ps + t9 / 3) * CW + wx * a.ps + t9 % 3) * SPITCH + ch * 16);
#pragma unroll
          for (int t9 = 0; t9 < 9; ++t9) {
            float v[8];
            Tr<bf16_t>::unpack(wv9[t9], v);
#pragma unroll
            for (int e = 0; e < 8; ++e) m[e] = fmx_raw(m[e], v[e]);
          }
        } else {
          for (int i = 0; i < a.pk; ++i)
            for (int j = 0; j < a.pk; ++j) {
              float v[8];
              Tr<bf16_t>::unpack(*(const u32x4_t*)(s_stage + ((wy * a.ps + i) * CW + wx * a.ps + j) * SPITCH + ch * 16), v);
#pragma unroll
              for (int e = 0; e < 8; ++e) m[e] = fmx_raw(m[e], v[e]);
            }
        }
        *(u32x4_t*)((unsigned char*)a.out + ((long long)n * a.out_sN + (long long)(py * a.PW + px) * a.out_sP) * 2 + ch * 16) = Tr<bf16_t>::pack(m);
      }
    } else {
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int it = 0; it < 32 / PPI; ++it) {
        const int px = it * PPI + lane / CPP, ch = lane % CPP;
        const u32x4_t o = *(const u32x4_t*)(stg + px * SPITCH + ch * 16);
        const int oy = cy0 + 2 * wave + (px >> 4), ox = cx0 + (px & 15);
        if (oy < a.OH && ox < a.OW)
          *(u32x4_t*)((unsigned char*)a.out + ((long long)n * a.out_sN + (long long)(oy * a.OW + ox) * a.out_sP) * 2 + ch * 16) = o;
      }
      __builtin_amdgcn_wave_barrier();
    }
    tile = next;
  }
}

template <int KB, bool POOL>
static int launch_stem_lds_kb(const ConvArgs& a, hipStream_t st) {
  const int taps = a.R * a.S;
  if (taps <= 12) hipLaunchKernelGGL((stem_lds_kernel<KB, 3, POOL>), dim3(a.grid), dim3(SL_NT), 0, st, a);
  else if (taps <= 28) hipLaunchKernelGGL((stem_lds_kernel<KB, 7, POOL>), dim3(a.grid), dim3(SL_NT), 0, st, a);
  else if (taps <= 52) hipLaunchKernelGGL((stem_lds_kernel<KB, 13, POOL>), dim3(a.grid), dim3(SL_NT), 0, st, a);
  else return (int)hipErrorInvalidValue;
  return (int)hipGetLastError();
}

static int launch_stem_lds(const ConvArgs& a, int dtype, hipStream_t st) {
  // the host checks what the kernel's LDS layout and indexing assume
  const bool pool = a.pool != POOL_NONE;
  const int CH = pool ? (a.pph - 1) * a.ps + a.pk : SL_TH, CW = pool ? (a.ppw - 1) * a.ps + a.pk : SL_TW;
  const int IH = (CH - 1) * a.stride + a.R, IW = (CW - 1) * a.stride + a.S;
  if (dtype != DT_BF16 || a.pair_C < 1 || a.pair_C > 4 || a.C != a.pair_C || a.R != a.S || a.R < 1 || a.R > 7 || (a.stride != 1 && a.stride != 2) ||
      a.pad < 0 || a.pad > a.R || IH * IW > stem_lds_in_positions(a.R * a.S) || IH >= 4096 || IW >= 4096 || !a.dw_w || a.has_res || a.ksplit >= 1 ||
      a.out_sK != 1 || a.out_f32 || (a.out_sP * 2) % 16 != 0 || (a.out_sN * 2) % 16 != 0 || ((uintptr_t)a.out & 15) || ((uintptr_t)a.dw_w & 15) ||
      a.pair_sN < 0 || a.pair_sC < 0 || a.pair_sH < 0 || (long long)4 * a.pair_sC + (long long)(a.H + 64) * a.pair_sH >= (1ll << 31) ||
      a.OH != (a.H + 2 * a.pad - a.R) / a.stride + 1 || a.OW != (a.W + 2 * a.pad - a.S) / a.stride + 1)
    return (int)hipErrorInvalidValue;
  if (pool) {
    // linked max-pooling: windows of 2 or 3, stride 2, padding 0 or 1; pph x ppw windows per tile whose convolution block
    // is at most 128 pixels; every window starts inside the map
    if (a.pool != POOL_MAX || a.pk < 2 || a.pk > 3 || a.ps != 2 || a.pp < 0 || a.pp > 1 || a.pph < 1 || a.ppw < 1 || CH * CW > 32 * SL_NW ||
        a.PH < 1 || a.PW < 1 || (a.PH - 1) * a.ps - a.pp >= a.OH || (a.PW - 1) * a.ps - a.pp >= a.OW ||
        a.tiles_y != (a.PH + a.pph - 1) / a.pph || a.tiles_x != (a.PW + a.ppw - 1) / a.ppw || a.tiles_m != a.N * a.tiles_y * a.tiles_x)
      return (int)hipErrorInvalidValue;
    if (a.K == 32) return launch_stem_lds_kb<1, true>(a, st);
    if (a.K == 64) return launch_stem_lds_kb<2, true>(a, st);
    return (int)hipErrorInvalidValue;
  }
  if (a.mode != M_FLAT || a.th != SL_TH || a.tw != SL_TW || a.tiles_y != (a.OH + SL_TH - 1) / SL_TH || a.tiles_x != (a.OW + SL_TW - 1) / SL_TW ||
      a.tiles_m != a.N * a.tiles_y * a.tiles_x)
    return (int)hipErrorInvalidValue;
  if (a.K == 32) return launch_stem_lds_kb<1, false>(a, st);
  if (a.K == 64) return launch_stem_lds_kb<2, false>(a, st);
  return (int)hipErrorInvalidValue;
}


template <typename T, int BM, int BN, int WM, int WN, bool SCALAR, int MODE>
static int launch_conv_inst(const ConvArgs& a, hipStream_t st) {
  constexpr int lds = lds_conv_bytes<BM, BN>();
  if (lds > 64 * 1024) {   // more than the default dynamic-LDS limit: raise it once per instantiation
    static bool raised = false;
    if (!raised) {
      hipError_t e = hipFuncSetAttribute((const void*)conv_kernel<T, BM, BN, WM, WN, SCALAR, MODE>,
                                         hipFuncAttributeMaxDynamicSharedMemorySize, lds);
      if (e != hipSuccess) return (int)e;
      raised = true;
    }
  }
  hipLaunchKernelGGL((conv_kernel<T, BM, BN, WM, WN, SCALAR, MODE>), dim3(a.grid), dim3(NT), lds, st, a);
  return (int)hipGetLastError();
}

template <typename T, int BM, int BN, int WM, int WN, bool SCALAR>
static int launch_conv_mode(const ConvArgs& a, hipStream_t st) {
  switch (a.mode) {
    case M_FLAT: return launch_conv_inst<T, BM, BN, WM, WN, SCALAR, M_FLAT>(a, st);
    case M_ZIGZAG: return launch_conv_inst<T, BM, BN, WM, WN, SCALAR, M_ZIGZAG>(a, st);
    case M_PATCH: return launch_conv_inst<T, BM, BN, WM, WN, SCALAR, M_PATCH>(a, st);
    case M_GAP: return launch_conv_inst<T, BM, BN, WM, WN, SCALAR, M_GAP>(a, st);
  }
  return (int)hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------------
// Depthwise -> pointwise chain with the depthwise result kept on chip (Section 2.2: the depthwise producer hands
// its output to the pointwise consumer in the consumer's channel-first order; here it never reaches memory).
// A workgroup owns 64 output pixels x 64 output channels.  Phase A computes the depthwise convolution
// (+ scale/shift + ReLU) of its 64 pixels for a whole panel of input channels straight into LDS, in the row-major
// [pixel][channel] form the GEMM reads, with every tap load of several pixels in flight at once, so the memory
// latency is paid once per panel rather than once per reduction step.  Phase B is the pointwise GEMM over the
// panel: A fragments come from the panel, weight tiles are double-buffered through registers.  The GEMM is
// computed transposed (accumulator rows = channels), the epilogue runs in registers and the finished tile goes
// through LDS once, in the output type, to be stored as 16-byte channel groups.
// Workgroups that share a pixel tile (different channel tiles) recompute its depthwise panel: 9 MACs per element
// against 64 per element and channel tile of the pointwise GEMM.
// ---------------------------------------------------------------------------------------------
__host__ __device__ constexpr int dwpw_panel_pitch(int cp, int esz) { return cp * esz + 16; }   // odd number of 16-byte slots
__host__ __device__ constexpr int dwpw_lds(int cp, int esz) { return 64 * dwpw_panel_pitch(cp, esz) + 2 * 64 * LDS_ROW; }

// (three wavefronts per SIMD: 143 registers instead of 167 + 16, a third workgroup per unit overlaps the two phases of
// the others; measured 2 % on a network of such chains at batch 32, four wavefronts spill and lose)
template <typename T>
__global__ __launch_bounds__(NT, 3) void dwpw_kernel(const ConvArgs a) {
  using tr = Tr<T>;
  constexpr int CE = tr::CE, BKE = tr::BKE, ESZ = (int)sizeof(T);
  constexpr int BM = 64, BN = 64;
  constexpr int B_IT = BN * CPR / NT;                              // 2 weight chunks per thread and step
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave >> 1, wave_n = wave & 1;                 // 2 x 2 wavefronts of 32 pixels x 32 channels
  const int l31 = lane & 31, lhalf = lane >> 5;

  const int CP = a.dw_panel;                                       // panel width in channels (multiple of BKE)
  const int PP = dwpw_panel_pitch(CP, ESZ);
  unsigned char* s_panel = smem;
  unsigned char* s_w = smem + BM * PP;
  const int OHW = a.OH * a.OW;
  const int Cpad = (a.C + BKE - 1) / BKE * BKE;                    // the packed weights are zero beyond C

  for (int t = blockIdx.x; t < a.ntiles; t += gridDim.x) {
    const int tile_m = t % a.tiles_m, tile_n = t / a.tiles_m;      // neighbours share a weight tile
    f32x16_t acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;

    for (int p0 = 0; p0 < Cpad; p0 += CP) {
      const int cp = Cpad - p0 < CP ? Cpad - p0 : CP;              // channels of this panel (multiple of BKE)
      const int cpc = cp / CE;                                     // 16-byte chunks per pixel
      // ---- phase A: depthwise chain of 64 pixels x cp channels into the panel -------------------------
      for (int it = tid; it < BM * cpc; it += NT) {
        const int px = it / cpc, c0 = p0 + (it - px * cpc) * CE;
        const int m = tile_m * BM + px;
        const bool valid = m < a.M_total && c0 < a.C;
        const int mm = m < a.M_total ? m : 0;
        const int n = mm / OHW, q = mm - n * OHW, oh = q / a.OW, ow = q - oh * a.OW;
        const int ih0 = oh * a.dw_stride - a.dw_pad, iw0 = ow * a.dw_stride - a.dw_pad;
        const long long base = (long long)n * a.dw_sN;
        const int cc = c0 < a.C ? c0 : 0;
        float d[CE];
#pragma unroll
        for (int e = 0; e < CE; ++e) d[e] = 0.f;
        if (a.dw_k == 3) {
          // all tap loads of the pixel are issued before any is used: one memory latency per pixel, not one per tap.
          // (Unrolling over several pixels and keeping the tap weights in registers was measured slower: the register
          // pressure costs more than the extra loads in flight gain.)  The phase is bound by its vector instructions
          // (460 per item, counted in the compiler's output, of which 72 multiplied masked taps by zero and 90 computed
          // nine 64-bit addresses from scratch): a masked tap reads a block of zeros instead, and a tap's address is the
          // window's first address plus a constant of the launch.
          u32x4_t xr[9], wr[9];
          const long long p00 = base + ((long long)ih0 * a.dw_W + iw0) * a.dw_sP + cc;   // (dereferenced only with an in-range tap)
          const long long rowst = (long long)a.dw_W * a.dw_sP;
          bool rok[3], cok[3];
#pragma unroll
          for (int j = 0; j < 3; ++j) {
            rok[j] = valid && (unsigned)(ih0 + j) < (unsigned)a.dw_H;
            cok[j] = (unsigned)(iw0 + j) < (unsigned)a.dw_W;
          }
#pragma unroll
          for (int t9 = 0; t9 < 9; ++t9) {
            const T* px = (const T*)a.in + p00 + (t9 / 3) * rowst + (t9 % 3) * a.dw_sP;
            xr[t9] = *(const u32x4_t*)((rok[t9 / 3] && cok[t9 % 3]) ? px : (const T*)a.zeros);
            wr[t9] = *(const u32x4_t*)((const T*)a.dw_w + (long long)t9 * a.C + cc);
          }
#pragma unroll
          for (int t9 = 0; t9 < 9; ++t9) {
            float x[CE], w[CE];
            tr::unpack(xr[t9], x);
            tr::unpack(wr[t9], w);
#pragma unroll
            for (int e = 0; e < CE; ++e) d[e] = fmaf(x[e], w[e], d[e]);
          }
        } else {
          for (int t9 = 0; t9 < a.dw_k * a.dw_k; ++t9) {
            const int ih = ih0 + t9 / a.dw_k, iw = iw0 + t9 % a.dw_k;
            const bool ok = valid && (unsigned)ih < (unsigned)a.dw_H && (unsigned)iw < (unsigned)a.dw_W;
            const long long off = ok ? base + ((long long)ih * a.dw_W + iw) * a.dw_sP + cc : cc;
            float x[CE], w[CE];
            tr::unpack(*(const u32x4_t*)((const T*)a.in + off), x);
            tr::unpack(*(const u32x4_t*)((const T*)a.dw_w + (long long)t9 * a.C + cc), w);
            const float keep = ok ? 1.f : 0.f;
#pragma unroll
            for (int e = 0; e < CE; ++e) d[e] = fmaf(x[e] * keep, w[e], d[e]);
          }
        }
        float sc[CE], sh[CE];
#pragma unroll
        for (int e = 0; e < CE; e += 4) {
          *(f32x4_t*)&sc[e] = *(const f32x4_t*)(a.dw_scale + cc + e);
          *(f32x4_t*)&sh[e] = *(const f32x4_t*)(a.dw_shift + cc + e);
        }
#pragma unroll
        for (int e = 0; e < CE; ++e) {
          float y = d[e] * sc[e] + sh[e];
          if (a.dw_relu) y = fmx(y, 0.f);
          d[e] = valid ? y : 0.f;                                  // rows past the end and padding channels are exact zeros
        }
        *(u32x4_t*)(s_panel + px * PP + (c0 - p0) * ESZ) = tr::pack(d);
      }
      // ---- phase B: pointwise GEMM over the panel --------------------------------------------------
      const int nst = cp / BKE, step0 = p0 / BKE;
      const unsigned char* wrow[B_IT];
#pragma unroll
      for (int it = 0; it < B_IT; ++it) {
        const int idx = tid + it * NT;
        wrow[it] = (const unsigned char*)a.w + ((long long)(tile_n * BN + idx / CPR) * a.Kred_pad + (idx % CPR) * CE) * (long long)ESZ +
                   (long long)step0 * ROWB;
      }
      u32x4_t rb0[B_IT], rb1[B_IT];
      auto load_w = [&](int s, u32x4_t* rb) {
        const int ss = s < nst ? s : nst - 1;                      // steps past the end re-read valid weights
#pragma unroll
        for (int it = 0; it < B_IT; ++it) rb[it] = *(const u32x4_t*)(wrow[it] + (long long)ss * ROWB);
      };
      auto store_w = [&](int stage, const u32x4_t* rb) {
#pragma unroll
        for (int it = 0; it < B_IT; ++it) {
          const int idx = tid + it * NT;
          *(u32x4_t*)(s_w + stage * BN * LDS_ROW + (idx / CPR) * LDS_ROW + (idx % CPR) * 16) = rb[it];
        }
      };
      auto compute = [&](int s, int stage) {
        const unsigned char* sa = s_panel + (wave_m * 32 + l31) * PP + s * ROWB + lhalf * 16;
        const unsigned char* sb = s_w + stage * BN * LDS_ROW + (wave_n * 32 + l31) * LDS_ROW + lhalf * 16;
#pragma unroll
        for (int kg = 0; kg < KG; ++kg) {
          const u32x4_t fa = *(const u32x4_t*)(sa + kg * 32), fb = *(const u32x4_t*)(sb + kg * 32);
          if constexpr (sizeof(T) == 2) {
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fb), __builtin_bit_cast(bf16x8_t, fa), acc, 0, 0, 0);
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fb[e]), __uint_as_float(fa[e]), acc, 0, 0, 0);
          }
        }
      };
      load_w(0, rb0);
      store_w(0, rb0);
      load_w(1, rb1);
      __syncthreads();                                             // panel and weight step 0 are visible
      for (int s = 0; s < nst; s += 2) {
        load_w(s + 2, rb0);
        compute(s, 0);
        store_w(1, rb1);
        __syncthreads();
        if (s + 1 >= nst) break;
        load_w(s + 3, rb1);
        compute(s + 1, 1);
        store_w(0, rb0);
        __syncthreads();
      }
      __syncthreads();                                             // everyone is done with the panel before it is overwritten
    }

    // ---- epilogue: lane = pixel wave_m*32 + l31, channels wave_n*32 + 8*g + 4*lhalf + (0..3) ---------------
    if (a.ksplit >= 1) {
      // the chain is finished by a summing pass (linked global average): hand it the raw fp32 sums
      const int m = tile_m * BM + wave_m * 32 + l31;
      if (m < a.M_total) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int k0 = tile_n * BN + wave_n * 32 + g * 8 + lhalf * 4;
          *(f32x4_t*)(a.part + (long long)m * a.part_ld + k0) = f32x4_t{acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]};
        }
      }
      continue;                                                    // uniform: no barrier is skipped by part of a workgroup
    }
    constexpr int SPB = BN * ESZ + 16;
    unsigned char* stg = s_panel;                                  // 64 rows x SPB bytes, inside the operand buffers
    const float lo = a.relu ? 0.f : -3.4028235e38f;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int c = wave_n * 32 + g * 8 + lhalf * 4, k0 = tile_n * BN + c;
      const f32x4_t sc = *(const f32x4_t*)(a.scale + k0), sh = *(const f32x4_t*)(a.shift + k0);
      float y[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) y[e] = fmx(acc[4 * g + e] * sc[e] + sh[e], lo);
      const int srow = wave_m * 32 + l31;
      if constexpr (sizeof(T) == 2) {
        uint2 o;
        o.x = f2bf2(y[0], y[1]);
        o.y = f2bf2(y[2], y[3]);
        *(uint2*)(stg + srow * SPB + c * 2) = o;
      } else {
        *(f32x4_t*)(stg + srow * SPB + c * 4) = f32x4_t{y[0], y[1], y[2], y[3]};
      }
    }
    __syncthreads();
    constexpr int CG = BN / CE;
    for (int idx = tid; idx < BM * CG; idx += NT) {
      const int r = idx / CG, cg = idx - r * CG;
      const int m = tile_m * BM + r, k0 = tile_n * BN + cg * CE;
      if (m >= a.M_total || k0 >= a.K) continue;
      const int n = m / OHW, q = m - n * OHW;
      const u32x4_t mine = *(const u32x4_t*)(stg + r * SPB + cg * 16);
      if (a.ileave)
        ileave_store<T>((T*)a.out + (long long)n * a.out_sN + (long long)q * a.out_sP + 2 * k0, mine,
                        *(const u32x4_t*)((const T*)a.res + (long long)n * a.res_sN + (long long)q * a.res_sP + k0), a.ileave == 1);
      else
        *(u32x4_t*)((T*)a.out + (long long)n * a.out_sN + (long long)q * a.out_sP + k0) = mine;
    }
    __syncthreads();
  }
}

template <typename T>
static int launch_dwpw_t(const ConvArgs& a, hipStream_t st) {
  constexpr int ESZ = (int)sizeof(T), BKE = Tr<T>::BKE, CE = Tr<T>::CE;
  const int lds = dwpw_lds(a.dw_panel, ESZ);
  // what the kernel assumes; anything else must take the general prologue path
  const bool raw = a.ksplit == 1 && a.part && a.part_ld >= a.tiles_n * 64 && a.part_ld % 4 == 0 && ((uintptr_t)a.part & 15) == 0;
  if (a.mode != M_FLAT || a.has_res || a.pool != POOL_NONE || (!a.vec_out && !raw) || (a.ksplit >= 1 && !raw) || a.kchunk || a.R != 1 || a.S != 1 || a.stride != 1 || a.pad != 0 ||
      a.C % CE != 0 || a.K % CE != 0 || a.dw_panel < BKE || a.dw_panel % BKE != 0 || lds > 160 * 1024 || a.dw_k < 1 ||
      a.tiles_m != (a.M_total + 63) / 64 || a.tiles_n != (a.K + 63) / 64 || a.ntiles != a.tiles_m * a.tiles_n || a.grid < 1 ||
      a.Kred_pad < (a.C + BKE - 1) / BKE * BKE || !a.dw_w || !a.dw_scale || !a.dw_shift || !a.zeros || ((uintptr_t)a.zeros & 15))
    return (int)hipErrorInvalidValue;
  static int raised = 0;
  if (lds > raised) {
    hipError_t e = hipFuncSetAttribute((const void*)dwpw_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return (int)e;
    raised = lds;
  }
  hipLaunchKernelGGL((dwpw_kernel<T>), dim3(a.grid < a.ntiles ? a.grid : a.ntiles), dim3(NT), lds, st, a);
  return (int)hipGetLastError();
}

template <typename T, int BM, int BN, int WM, int WN, int MODE>
static int launch_conv_dwpro_inst(const ConvArgs& a, hipStream_t st) {
  constexpr int lds = lds_conv_bytes<BM, BN>();
  static bool raised = false;
  if (lds > 64 * 1024 && !raised) {
    hipError_t e = hipFuncSetAttribute((const void*)conv_kernel<T, BM, BN, WM, WN, false, MODE, true>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return (int)e;
    raised = true;
  }
  hipLaunchKernelGGL((conv_kernel<T, BM, BN, WM, WN, false, MODE, true>), dim3(a.grid), dim3(NT), lds, st, a);
  return (int)hipGetLastError();
}

// linked depthwise -> pointwise chain: 1x1 / stride 1 / pad 0 consumer, FLAT or GAP rows, 64x64 tile
template <typename T>
static int launch_conv_dwpro_t(const ConvArgs& a, int cfg, hipStream_t st) {
  if (a.R != 1 || a.S != 1 || a.stride != 1 || a.pad != 0 || a.kchunk || a.C % Tr<T>::CE != 0 || !a.dw_w || a.dw_k < 1)
    return (int)hipErrorInvalidValue;
  if (cfg == 2 && a.dw_panel > 0) return launch_dwpw_t<T>(a, st);       // depthwise panel on chip
  if (cfg == 2 && a.mode == M_FLAT) return launch_conv_dwpro_inst<T, 64, 64, 32, 32, M_FLAT>(a, st);
  if (cfg == 2 && a.mode == M_GAP) return launch_conv_dwpro_inst<T, 64, 64, 32, 32, M_GAP>(a, st);
  return (int)hipErrorInvalidValue;
}

template <typename T>
static int launch_conv_t(const ConvArgs& a, int cfg, int scalar, hipStream_t st) {
  if (scalar) {   // the element-wise gather loader (odd channel counts, strided graph input) exists for the 64x64 tile only
    if (cfg == 2) return launch_conv_mode<T, 64, 64, 32, 32, true>(a, st);
    return (int)hipErrorInvalidValue;
  }
  switch (cfg) {
    case 0: return launch_conv_mode<T, 128, 128, 64, 64, false>(a, st);
    case 1: return launch_conv_mode<T, 128, 64, 64, 32, false>(a, st);
    case 2: return launch_conv_mode<T, 64, 64, 32, 32, false>(a, st);
    case 3: return launch_conv_mode<T, 32, 128, 32, 32, false>(a, st);
  }
  return (int)hipErrorInvalidValue;
}

int launch_conv(const ConvArgs& a, int dtype, int cfg, int scalar_loader, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  if (a.grid < 1 || a.tiles_m < 1 || a.tiles_n < 1) return (int)hipErrorInvalidValue;
  if (cfg < kHaloCfg && a.xcd_m != 1 && a.xcd_m != 2 && a.xcd_m != 4 && a.xcd_m != 8) return (int)hipErrorInvalidValue;
  if (a.ksplit >= 1 && (a.mode != M_FLAT || !a.part || a.steps_per_split < 1 || (a.dw_w && a.dw_panel <= 0))) return (int)hipErrorInvalidValue;
  if (a.ileave) {
    // the interleaving store exists in the pixel-major epilogues of the general kernel and of the depthwise-panel kernel;
    // it moves whole 16-byte groups
    const int ce = dtype == DT_BF16 ? 8 : 4, esz = dtype == DT_BF16 ? 2 : 4;
    if (cfg >= kHaloCfg || a.mode != M_FLAT || a.has_res || a.ksplit >= 1 || a.pair || !a.res || a.out_f32 || a.out_sK != 1 ||
        (a.ileave != 1 && a.ileave != 2) || a.K % ce != 0 || a.out_sP % ce != 0 || a.out_sN % ce != 0 || a.res_sP % ce != 0 || a.res_sN % ce != 0 ||
        ((uintptr_t)a.out % 16) != 0 || ((uintptr_t)a.res % 16) != 0 || a.out_sP < 2 * a.K || a.res_sP < a.K || esz * ce != 16)
      return (int)hipErrorInvalidValue;
  }
  if (cfg == kPairCfg || a.pair) {
    if (cfg != kPairCfg || scalar_loader) return (int)hipErrorInvalidValue;
    return launch_pair(a, dtype, st);
  }
  if (cfg == kFcCfg) {
    if (scalar_loader) return (int)hipErrorInvalidValue;
    return launch_fc(a, dtype, st);
  }
  if (cfg == kStemLdsCfg) return launch_stem_lds(a, dtype, st);
  if (cfg == kFireCfg || a.fire) {
    if (cfg != kFireCfg || !a.fire || scalar_loader) return (int)hipErrorInvalidValue;
    return launch_fire(a, dtype, st);
  }
  if (cfg == kPwDwCfg || a.pwdw) {
    if (cfg != kPwDwCfg || !a.pwdw || scalar_loader) return (int)hipErrorInvalidValue;
    return launch_pwdw(a, dtype, st);
  }
  if (a.dw_w) {
    if (scalar_loader) return (int)hipErrorInvalidValue;
    return dtype == DT_BF16 ? launch_conv_dwpro_t<bf16_t>(a, cfg, st) : launch_conv_dwpro_t<float>(a, cfg, st);
  }
  if (cfg == kHaloCfg) {
    if (a.halo_mgroup < 1) return (int)hipErrorInvalidValue;
    if (scalar_loader) return (int)hipErrorInvalidValue;
    return dtype == DT_BF16 ? launch_conv3x3_t<bf16_t>(a, st) : launch_conv3x3_t<float>(a, st);
  }
  if (cfg == kStemCfg) return dtype == DT_BF16 ? launch_stem_t<bf16_t>(a, st) : launch_stem_t<float>(a, st);
  return dtype == DT_BF16 ? launch_conv_t<bf16_t>(a, cfg, scalar_loader, st) : launch_conv_t<float>(a, cfg, scalar_loader, st);
}

size_t conv_lds_bytes(int cfg, int /*mode*/) {
  if (cfg == kHaloCfg) return v2_lds_total(128);
  if (cfg == kPairCfg) return PR_LDS;
  if (cfg == kFcCfg) return 0;
  if (cfg == kStemLdsCfg) return 32 * 1024;   // static: input block, staging slices, tables
  if (cfg == kStemCfg) return 40 * 1024;   // static: staging slices (at most 4 x 32 x 272 bytes) + tables
  const TileCfg& c = kTileCfgs[cfg];
  const size_t main_b = (size_t)2 * (c.bm + c.bn) * LDS_ROW;
  const size_t stg_b = (size_t)c.bm * (c.bn + STG_PAD) * 4;
  return stg_b > main_b ? stg_b : main_b;
}

bool conv_cfg_has_scalar_loader(int cfg) { return cfg == 2; }
bool conv_cfg_has_dw_prologue(int cfg, int mode) { return cfg == 2 && (mode == M_FLAT || mode == M_GAP); }
size_t dwpw_lds_bytes(int panel_channels, int esz) { return (size_t)dwpw_lds(panel_channels, esz); }

// ---------------------------------------------------------------------------------------------
// Depthwise convolution chain: one thread = one 16-byte channel vector of one output pixel.
// ---------------------------------------------------------------------------------------------
// K3: the 3x3 kernel with its nine taps unrolled; IDX = int when the work items fit 31 bits (three 32-bit divisions per
// item instead of three 64-bit ones, which cost more than the nine taps).
template <typename T, bool K3, typename IDX>
__global__ __launch_bounds__(NT) void dw_kernel(const DwArgs a) {
  using tr = Tr<T>;
  constexpr int CE = tr::CE;
  const int cv = a.C / CE;
  const int R = K3 ? 3 : a.R, S = K3 ? 3 : a.S;
  for (IDX idx = (IDX)blockIdx.x * NT + threadIdx.x; idx < (IDX)a.total_vec; idx += (IDX)gridDim.x * NT) {
    const int c0 = (int)(idx % cv) * CE;
    IDX pix = idx / cv;
    const int ow = (int)(pix % a.OW); pix /= a.OW;
    const int oh = (int)(pix % a.OH);
    const int n = (int)(pix / a.OH);
    float acc[CE];
#pragma unroll
    for (int e = 0; e < CE; ++e) acc[e] = 0.f;
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int ih = oh * a.stride - a.pad + r;
      if ((unsigned)ih >= (unsigned)a.H) continue;
#pragma unroll
      for (int s = 0; s < S; ++s) {
        const int iw = ow * a.stride - a.pad + s;
        if ((unsigned)iw >= (unsigned)a.W) continue;
        const T* p = (const T*)a.in + (long long)n * a.in_sN + ((long long)ih * a.W + iw) * a.in_sP + c0;
        const T* q = (const T*)a.w + (long long)(r * S + s) * a.C + c0;
        float x[CE], w[CE];
        tr::unpack(*(const u32x4_t*)p, x);
        tr::unpack(*(const u32x4_t*)q, w);
#pragma unroll
        for (int e = 0; e < CE; ++e) acc[e] = fmaf(x[e], w[e], acc[e]);
      }
    }
#pragma unroll
    for (int e = 0; e < CE; ++e) {
      float v = acc[e] * a.scale[c0 + e] + a.shift[c0 + e];
      acc[e] = a.relu ? fmx(v, 0.f) : v;
    }
    T* o = (T*)a.out + (long long)n * a.out_sN + ((long long)oh * a.OW + ow) * a.out_sP + c0;
    *(u32x4_t*)o = tr::pack(acc);
  }
}

static int grid_for(long long work_items, int per_block) {
  long long b = (work_items + per_block - 1) / per_block;
  if (b < 1) b = 1;
  if (b > 256 * 32) b = 256 * 32;
  return (int)b;
}

int launch_dw(const DwArgs& a, int dtype, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  const int grid = grid_for(a.total_vec, NT);
  if (a.total_vec < 0 || a.R < 1 || a.S < 1) return (int)hipErrorInvalidValue;
  const bool k3 = a.R == 3 && a.S == 3;
  const bool small = a.total_vec + (long long)grid * NT < (1ll << 31);   // (the grid-stride loop steps past the end once)
  if (dtype == DT_BF16) {
    if (k3 && small) hipLaunchKernelGGL((dw_kernel<bf16_t, true, int>), dim3(grid), dim3(NT), 0, st, a);
    else if (small) hipLaunchKernelGGL((dw_kernel<bf16_t, false, int>), dim3(grid), dim3(NT), 0, st, a);
    else hipLaunchKernelGGL((dw_kernel<bf16_t, false, long long>), dim3(grid), dim3(NT), 0, st, a);
  } else {
    if (k3 && small) hipLaunchKernelGGL((dw_kernel<float, true, int>), dim3(grid), dim3(NT), 0, st, a);
    else if (small) hipLaunchKernelGGL((dw_kernel<float, false, int>), dim3(grid), dim3(NT), 0, st, a);
    else hipLaunchKernelGGL((dw_kernel<float, false, long long>), dim3(grid), dim3(NT), 0, st, a);
  }
  return (int)hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Second half of a reduction-split chain: sum the shares in index order, then scale/shift, shortcut, ReLU, store.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(NT) void splitk_finish_kernel(const SplitKArgs a) {
  using tr = Tr<T>;
  // the shares of one output element, added in index order.  Eight loads are requested before the first is added: a
  // loop of load-then-add pays one cache latency per share (32 shares: 5 us for the plain pass, 20 us for the averaging
  // one, measured), this pays one per eight.
  auto sum_shares = [&](const float* p0) __attribute__((always_inline)) -> float {
    const long long zs = (long long)a.M * a.part_ld;
    float v = 0.f;
    int z = 0;
    for (; z + 8 <= a.ksplit; z += 8) {
      float t[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) t[u] = p0[(z + u) * zs];
#pragma unroll
      for (int u = 0; u < 8; ++u) v += t[u];
    }
    if (z + 4 <= a.ksplit) {
      float t[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) t[u] = p0[(z + u) * zs];
#pragma unroll
      for (int u = 0; u < 4; ++u) v += t[u];
      z += 4;
    }
    for (; z < a.ksplit; ++z) v += p0[z * zs];
    return v;
  };
  if (a.gap) {
    // linked global average (CBRA): a workgroup owns 16 channels of one image; 16 thread groups finish the pixels
    // p = g, g + 16, ... and the 16 partial sums are added in group order
    constexpr int CH = 16, PG = NT / CH;
    __shared__ float s_sum[NT];
    const int kt = (a.K + CH - 1) / CH;
    const int kk = threadIdx.x % CH, pg = threadIdx.x / CH;
    for (int blk = blockIdx.x; blk < (a.M / a.OHW) * kt; blk += gridDim.x) {
      const long long n = blk / kt;
      const int k = (blk % kt) * CH + kk;
      float s = 0.f;
      if (k < a.K) {
        const float sc = a.scale[k], sh = a.shift[k];
        for (int p = pg; p < a.OHW; p += PG) {
          const long long m = n * a.OHW + p;
          float v = sum_shares(a.part + m * a.part_ld + k);
          v = v * sc + sh;
          if (a.res) v += tr::ld(a.res, n * a.res_sN + p * a.res_sP + k);
          if (a.relu) v = fmx(v, 0.f);
          s += v;
        }
      }
      s_sum[threadIdx.x] = s;
      __syncthreads();
      if (pg == 0 && k < a.K) {
        float t = 0.f;
        for (int w = 0; w < PG; ++w) t += s_sum[w * CH + kk];
        t /= (float)a.OHW;
        const long long o = n * a.out_sN + (long long)k * a.out_sK;
        if (a.out_f32) ((float*)a.out)[o] = t; else tr::st(a.out, o, t);
      }
      __syncthreads();
    }
    return;
  }
  const long long total = (long long)a.M * a.K;
  for (long long idx = (long long)blockIdx.x * NT + threadIdx.x; idx < total; idx += (long long)gridDim.x * NT) {
    const int k = (int)(idx % a.K);
    const long long m = idx / a.K;
    float v = sum_shares(a.part + m * a.part_ld + k);
    v = v * a.scale[k] + a.shift[k];
    const long long n = m / a.OHW, p = m - n * a.OHW;
    if (a.res) v += tr::ld(a.res, n * a.res_sN + p * a.res_sP + k);
    if (a.relu) v = fmx(v, 0.f);
    const long long o = n * a.out_sN + p * a.out_sP + (long long)k * a.out_sK;
    if (a.out_f32) ((float*)a.out)[o] = v; else tr::st(a.out, o, v);
  }
}

int launch_splitk_finish(const SplitKArgs& a, int dtype, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  if (a.ksplit < 1 || a.OHW < 1 || a.M % a.OHW != 0) return (int)hipErrorInvalidValue;
  const int grid = a.gap ? grid_for((long long)(a.M / a.OHW) * ((a.K + 15) / 16), 1) : grid_for((long long)a.M * a.K, NT);
  if (dtype == DT_BF16) hipLaunchKernelGGL(splitk_finish_kernel<bf16_t>, dim3(grid), dim3(NT), 0, st, a);
  else hipLaunchKernelGGL(splitk_finish_kernel<float>, dim3(grid), dim3(NT), 0, st, a);
  return (int)hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Stand-alone element-wise pass (bias / BN as scale+shift, ReLU, add, concat copy) on NHWC views.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(NT) void elt_kernel(const EltArgs a) {
  using tr = Tr<T>;
  const long long total = a.pixels * a.C;
  for (long long idx = (long long)blockIdx.x * NT + threadIdx.x; idx < total; idx += (long long)gridDim.x * NT) {
    const int c = (int)(idx % a.C);
    const long long p = idx / a.C;
    float v = tr::ld(a.a, p * a.a_sP + c * a.a_sK);
    if (a.op == ELT_AFFINE) v = v * a.scale[c] + a.shift[c];
    else if (a.op == ELT_ADD) v += tr::ld(a.b, p * a.b_sP + c);
    if (a.relu || a.op == ELT_RELU) v = fmx(v, 0.f);
    tr::st(a.out, p * a.out_sP + c * a.out_sK, v);
  }
}

template <typename T>
__global__ __launch_bounds__(NT) void elt_vec_kernel(const EltArgs a) {
  using tr = Tr<T>;
  constexpr int CE = tr::CE;
  const int cv = a.C / CE;
  const long long total = a.pixels * cv;
  for (long long idx = (long long)blockIdx.x * NT + threadIdx.x; idx < total; idx += (long long)gridDim.x * NT) {
    const int c = (int)(idx % cv) * CE;
    const long long p = idx / cv;
    float v[CE];
    tr::unpack(*(const u32x4_t*)((const T*)a.a + p * a.a_sP + c), v);
    if (a.op == ELT_AFFINE) {
#pragma unroll
      for (int e = 0; e < CE; ++e) v[e] = v[e] * a.scale[c + e] + a.shift[c + e];
    } else if (a.op == ELT_ADD) {
      float w[CE];
      tr::unpack(*(const u32x4_t*)((const T*)a.b + p * a.b_sP + c), w);
#pragma unroll
      for (int e = 0; e < CE; ++e) v[e] += w[e];
    }
    if (a.relu || a.op == ELT_RELU) {
#pragma unroll
      for (int e = 0; e < CE; ++e) v[e] = fmx(v[e], 0.f);
    }
    *(u32x4_t*)((T*)a.out + p * a.out_sP + c) = tr::pack(v);
  }
}

int launch_elt(const EltArgs& a, int dtype, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  const int ce = dtype == DT_BF16 ? 8 : 4;
  if (a.a_sK < 1 || a.out_sK < 1) return (int)hipErrorInvalidValue;
  const bool vec = a.a_sK == 1 && a.out_sK == 1 && a.C % ce == 0 && a.a_sP % ce == 0 && a.out_sP % ce == 0 && (a.op != ELT_ADD || a.b_sP % ce == 0) &&
                   ((uintptr_t)a.a % 16 == 0) && ((uintptr_t)a.out % 16 == 0) && (a.op != ELT_ADD || (uintptr_t)a.b % 16 == 0);
  if (vec) {
    const int grid = grid_for(a.pixels * (a.C / ce), NT);
    if (dtype == DT_BF16) hipLaunchKernelGGL(elt_vec_kernel<bf16_t>, dim3(grid), dim3(NT), 0, st, a);
    else hipLaunchKernelGGL(elt_vec_kernel<float>, dim3(grid), dim3(NT), 0, st, a);
  } else {
    const int grid = grid_for(a.pixels * a.C, NT);
    if (dtype == DT_BF16) hipLaunchKernelGGL(elt_kernel<bf16_t>, dim3(grid), dim3(NT), 0, st, a);
    else hipLaunchKernelGGL(elt_kernel<float>, dim3(grid), dim3(NT), 0, st, a);
  }
  return (int)hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Stand-alone pooling pass (max / average / global average) on NHWC views; one thread per output element.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(NT) void pool_kernel(const PoolArgs a) {
  using tr = Tr<T>;
  const long long total = (long long)a.N * a.OH * a.OW * a.C;
  for (long long idx = (long long)blockIdx.x * NT + threadIdx.x; idx < total; idx += (long long)gridDim.x * NT) {
    const int c = (int)(idx % a.C);
    long long q = idx / a.C;
    const int ow = (int)(q % a.OW); q /= a.OW;
    const int oh = (int)(q % a.OH);
    const int n = (int)(q / a.OH);
    const long long ib = (long long)n * a.in_sN + c;
    float r;
    if (a.kind == POOL_GAP) {
      float s = 0.f;
      for (int p = 0; p < a.H * a.W; ++p) s += tr::ld(a.in, ib + (long long)p * a.in_sP);
      r = s / (float)(a.H * a.W);
    } else {
      float mx = -INFINITY, sum = 0.f;
      int cnt = 0, cntp = 0;
      for (int i = 0; i < a.k; ++i)
        for (int j = 0; j < a.k; ++j) {
          const int ih = oh * a.s - a.p + i, iw = ow * a.s - a.p + j;
          if (ih < a.H + a.p && iw < a.W + a.p) ++cntp;
          if (ih < 0 || ih >= a.H || iw < 0 || iw >= a.W) continue;
          const float v = tr::ld(a.in, ib + ((long long)ih * a.W + iw) * a.in_sP);
          mx = fmx_raw(mx, v); sum += v; ++cnt;
        }
      r = a.kind == POOL_MAX ? mx : sum / (float)(a.cip ? cntp : cnt);
    }
    tr::st(a.out, (long long)n * a.out_sN + ((long long)oh * a.OW + ow) * a.out_sP + c, r);
  }
}

// Window pooling over whole 16-byte channel groups: one thread = one channel group of one output pixel.
template <typename T>
__global__ __launch_bounds__(NT) void pool_vec_kernel(const PoolArgs a) {
  using tr = Tr<T>;
  constexpr int CE = tr::CE;
  const int CV = a.C / CE;
  const long long total = (long long)a.N * a.OH * a.OW * CV;
  for (long long idx = (long long)blockIdx.x * NT + threadIdx.x; idx < total; idx += (long long)gridDim.x * NT) {
    const int cv = (int)(idx % CV);
    long long q = idx / CV;
    const int ow = (int)(q % a.OW); q /= a.OW;
    const int oh = (int)(q % a.OH);
    const int n = (int)(q / a.OH);
    const T* ib = (const T*)a.in + (long long)n * a.in_sN + cv * CE;
    float mx[CE], sum[CE];
#pragma unroll
    for (int e = 0; e < CE; ++e) { mx[e] = -INFINITY; sum[e] = 0.f; }
    int cnt = 0, cntp = 0;
    // windows of 2x2 and 3x3: every element of the window is requested before the first is used (elements outside the map
    // read the image's first pixel and are skipped); as a loop over rows and columns the pass paid one memory latency per
    // element of the window
    auto window = [&](auto kc) __attribute__((always_inline)) {
      constexpr int K = decltype(kc)::value;
      u32x4_t wv[K * K];
      unsigned in = 0;
#pragma unroll
      for (int t = 0; t < K * K; ++t) {
        const int ih = oh * a.s - a.p + t / K, iw = ow * a.s - a.p + t % K;
        if (ih < a.H + a.p && iw < a.W + a.p) ++cntp;
        const bool ok = ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
        in |= (ok ? 1u : 0u) << t;
        wv[t] = *(const u32x4_t*)(ib + (ok ? ((long long)ih * a.W + iw) * a.in_sP : 0));
      }
#pragma unroll
      for (int t = 0; t < K * K; ++t) {
        if (!((in >> t) & 1u)) continue;
        float v[CE];
        tr::unpack(wv[t], v);
#pragma unroll
        for (int e = 0; e < CE; ++e) { mx[e] = fmx_raw(mx[e], v[e]); sum[e] += v[e]; }
        ++cnt;
      }
    };
    if (a.k == 3) window(std::integral_constant<int, 3>{});
    else if (a.k == 2) window(std::integral_constant<int, 2>{});
    else
    for (int i = 0; i < a.k; ++i)
      for (int j = 0; j < a.k; ++j) {
        const int ih = oh * a.s - a.p + i, iw = ow * a.s - a.p + j;
        if (ih < a.H + a.p && iw < a.W + a.p) ++cntp;
        if (ih < 0 || ih >= a.H || iw < 0 || iw >= a.W) continue;
        float v[CE];
        tr::unpack(*(const u32x4_t*)(ib + ((long long)ih * a.W + iw) * a.in_sP), v);
#pragma unroll
        for (int e = 0; e < CE; ++e) { mx[e] = fmx_raw(mx[e], v[e]); sum[e] += v[e]; }
        ++cnt;
      }
    float r[CE];
    const float div = (float)(a.cip ? cntp : cnt);
#pragma unroll
    for (int e = 0; e < CE; ++e) r[e] = a.kind == POOL_MAX ? mx[e] : sum[e] / div;
    *(u32x4_t*)((T*)a.out + (long long)n * a.out_sN + ((long long)oh * a.OW + ow) * a.out_sP + cv * CE) = tr::pack(r);
  }
}

int launch_pool(const PoolArgs& a, int dtype, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  const int ce = dtype == DT_BF16 ? 8 : 4, esz = dtype == DT_BF16 ? 2 : 4;
  const bool vec = a.kind != POOL_GAP && a.C % ce == 0 && a.in_sP % ce == 0 && a.in_sN % ce == 0 && a.out_sP % ce == 0 &&
                   a.out_sN % ce == 0 && ((uintptr_t)a.in & 15) == 0 && ((uintptr_t)a.out & 15) == 0 && esz > 0;
  if (vec) {
    const int grid = grid_for((long long)a.N * a.OH * a.OW * (a.C / ce), NT);
    if (dtype == DT_BF16) hipLaunchKernelGGL(pool_vec_kernel<bf16_t>, dim3(grid), dim3(NT), 0, st, a);
    else hipLaunchKernelGGL(pool_vec_kernel<float>, dim3(grid), dim3(NT), 0, st, a);
    return (int)hipGetLastError();
  }
  const int grid = grid_for((long long)a.N * a.OH * a.OW * a.C, NT);
  if (dtype == DT_BF16) hipLaunchKernelGGL(pool_kernel<bf16_t>, dim3(grid), dim3(NT), 0, st, a);
  else hipLaunchKernelGGL(pool_kernel<float>, dim3(grid), dim3(NT), 0, st, a);
  return (int)hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Graph-boundary layout / type conversion (strided gather, channel-fastest writes).
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(NT) void cvt_kernel(const CvtArgs a) {
  using tr = Tr<T>;
  const long long HW = (long long)a.H * a.W, total = (long long)a.N * HW * a.Cout;
  for (long long idx = (long long)blockIdx.x * NT + threadIdx.x; idx < total; idx += (long long)gridDim.x * NT) {
    const int c = (int)(idx % a.Cout);
    long long q = idx / a.Cout;
    const long long p = q % HW;
    const long long n = q / HW;
    const long long o = n * a.out_sN + c * a.out_sC + p * a.out_sP;
    float v = 0.f;                                                 // padding channel
    if (c < a.C) {
      const long long i = n * a.in_sN + c * a.in_sC + p * a.in_sP;
      v = a.in_f32 ? ((const float*)a.in)[i] : tr::ld(a.in, i);
    }
    if (a.out_f32) ((float*)a.out)[o] = v; else tr::st(a.out, o, v);
  }
}

int launch_cvt(const CvtArgs& a, int dtype, void* stream) {
  hipStream_t st = (hipStream_t)stream;
  const int grid = grid_for((long long)a.N * a.H * a.W * a.Cout, NT);
  if (dtype == DT_BF16) hipLaunchKernelGGL(cvt_kernel<bf16_t>, dim3(grid), dim3(NT), 0, st, a);
  else hipLaunchKernelGGL(cvt_kernel<float>, dim3(grid), dim3(NT), 0, st, a);
  return (int)hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Micro-kernels that measure what this device attains, for the denominators of the roofline report:
// an MFMA-only loop (no memory instruction in the loop) and a streaming read of device memory.
// ---------------------------------------------------------------------------------------------
constexpr int PROBE_WG_PER_CU = 2;

// `data` selects the operand values, which decide the rate: the chip lowers its clock with the switching activity of the
// MFMA inputs.  0 = a handful of small values per lane (little toggling), 1 = pseudo-random dense operands (random sign,
// mantissa and a 2-bit exponent spread, the weight operand 16 times smaller), 2 = the same with every second pixel-operand
// element zero, as activations behind a ReLU are.  Four fragments per operand rotate through eight accumulators.
__global__ __launch_bounds__(NT) void probe_mfma_kernel(float* out, int iters, int data) {
  const int lane = threadIdx.x & 63;
  bf16x8_t fa[4], fb[4];
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      if (data == 0) {
        fa[s][e] = (__bf16)(0.001f * (float)((lane + e + s) & 7));
        fb[s][e] = (__bf16)(0.002f * (float)((lane * 3 + e + s) & 7));
      } else {
        uint32_t h = (uint32_t)lane * 2654435761u ^ (uint32_t)(s * 8 + e + 1) * 0x9E3779B9u;
        h ^= h >> 16; h *= 0x7feb352du; h ^= h >> 15; h *= 0x846ca68bu; h ^= h >> 16;
        const uint32_t sign = h & 1u, mant = (h >> 1) & 0x7fu, ex = 124u + ((h >> 8) & 3u);
        const bool zero = data == 2 && ((h >> 12) & 1u);
        const uint16_t va = zero ? (uint16_t)0 : (uint16_t)((sign << 15) | (ex << 7) | mant);
        const uint32_t g = h * 0x2c1b3c6du + 0x297a2d39u;
        const uint16_t vb = (uint16_t)(((g & 1u) << 15) | ((120u + ((g >> 8) & 3u)) << 7) | ((g >> 1) & 0x7fu));
        fa[s][e] = __builtin_bit_cast(__bf16, va);
        fb[s][e] = __builtin_bit_cast(__bf16, vb);
      }
    }
  f32x16_t acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
  for (int i = 0; i < iters; i += 4) {
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[(j + k) & 3], fa[((j >> 2) + k) & 3], acc[j], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) sum += acc[j][e];
  out[(size_t)blockIdx.x * NT + threadIdx.x] = sum;
}

__global__ __launch_bounds__(NT) void probe_read_kernel(const u32x4_t* in, size_t n16, uint32_t* out) {
  uint32_t x = 0;
  const size_t stride = (size_t)gridDim.x * NT;
  size_t i = (size_t)blockIdx.x * NT + threadIdx.x;
  // four loads in flight per thread
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4_t a = in[i], b = in[i + stride], c = in[i + 2 * stride], d = in[i + 3 * stride];
    x ^= a[0] ^ a[1] ^ a[2] ^ a[3] ^ b[0] ^ b[1] ^ b[2] ^ b[3] ^ c[0] ^ c[1] ^ c[2] ^ c[3] ^ d[0] ^ d[1] ^ d[2] ^ d[3];
  }
  for (; i < n16; i += stride) { const u32x4_t a = in[i]; x ^= a[0] ^ a[1] ^ a[2] ^ a[3]; }
  out[(size_t)blockIdx.x * NT + threadIdx.x] = x;
}

// MFMA loop on every compute unit: returns the floating-point operations the launch performs through *flops.
// d_out must hold probe_out_bytes(num_cu) bytes.
int launch_probe_mfma(void* d_out, int num_cu, int iters, int data, void* stream, double* flops) {
  if (!d_out || num_cu < 1 || iters < 1 || data < 0 || data > 2) return (int)hipErrorInvalidValue;
  iters = (iters + 3) / 4 * 4;                                     // (the loop runs four rounds per turn)
  const int grid = num_cu * PROBE_WG_PER_CU;
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(grid), dim3(NT), 0, (hipStream_t)stream, (float*)d_out, iters, data);
  if (flops) *flops = (double)grid * (NT / 64) * (double)iters * 8.0 * (2.0 * 32 * 32 * 16);
  return (int)hipGetLastError();
}

// streaming read of `bytes` (a multiple of 16) from d_in; d_out must hold probe_out_bytes(num_cu) bytes
int launch_probe_read(const void* d_in, size_t bytes, void* d_out, int num_cu, void* stream) {
  if (!d_in || !d_out || num_cu < 1 || bytes < 16 || (bytes & 15) || ((uintptr_t)d_in & 15)) return (int)hipErrorInvalidValue;
  const int grid = num_cu * 8;
  hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(NT), 0, (hipStream_t)stream, (const u32x4_t*)d_in, bytes / 16, (uint32_t*)d_out);
  return (int)hipGetLastError();
}

size_t probe_out_bytes(int num_cu) { return (size_t)num_cu * 8 * NT * 4; }

}  // namespace xenos
