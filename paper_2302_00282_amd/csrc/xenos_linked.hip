// gfx950 (CDNA4) kernels of the chains whose intermediate tensor stays on chip between two convolutions
// (Table 1, ConvX -> ConvY; Section 2.2 and the last paragraph of Section 4.1):
//
//  pwdw_kernel   pointwise (1x1) convolution chain -> depthwise 3x3 convolution chain.  The pointwise output of a
//                spatial tile plus the one-pixel halo the depthwise windows need lives in LDS only, written there by
//                the GEMM epilogue in the [position][channel] order the depthwise stencil reads.
#include "device_common.h"

namespace xenos {

// ---------------------------------------------------------------------------------------------
// Pointwise -> depthwise on chip.
//
// The paper's motivating mismatch (Section 2.2): a producer that writes in one order and a consumer that reads in
// another.  Here the pointwise output never reaches memory at all.  A depthwise convolution works per channel, so
// the pair splits over output channels first (Section 4.2.1) with no redundancy: a workgroup owns a TH x TW block
// of depthwise OUTPUT pixels of one image x 64 channels.  It computes the pointwise chain (GEMM over all input
// channels + scale/shift + ReLU) for the ((TH-1)*s+3) x ((TW-1)*s+3) block of pixels those windows cover, in
// chunks of 64 pixels, straight into an LDS block in the storage type (rounded as a stored tensor would be); block
// positions outside the map stay zero, they are the depthwise padding.  Neighbouring tiles recompute the shared
// border (the paper's halo replication).  Then every thread runs the nine taps of one 16-byte channel group of one
// output pixel out of LDS, applies the depthwise chain's scale/shift/ReLU and stores 16 bytes.
//
// GEMM: 4 wavefronts as 2 x 2 of 32 pixels x 32 channels, operands double-buffered through registers and LDS,
// computed transposed (accumulator rows = channels) so that a lane holds 4 consecutive channels of one pixel.
// ---------------------------------------------------------------------------------------------
constexpr int PD_BM = 64, PD_BN = kPwDwChannels;
__host__ __device__ constexpr int pwdw_mid_pitch(int esz) { return PD_BN * esz + 16; }   // an odd number of 16-byte slots
__host__ __device__ constexpr int pwdw_lds(int positions, int esz) { return positions * pwdw_mid_pitch(esz) + 2 * (PD_BM + PD_BN) * LDS_ROW; }

template <typename T>
__global__ __launch_bounds__(NT) void pwdw_kernel(const ConvArgs a) {
  using tr = Tr<T>;
  constexpr int CE = tr::CE, BKE = tr::BKE, ESZ = (int)sizeof(T);
  constexpr int BM = PD_BM, BN = PD_BN;
  constexpr int MP = pwdw_mid_pitch(ESZ);
  constexpr int CG = BN / CE;                                      // 16-byte channel groups of a position
  constexpr int A_IT = BM * CPR / NT, B_IT = BN * CPR / NT;        // 16-byte chunks per thread and step
  static_assert(A_IT >= 1 && B_IT >= 1 && NT % CG == 0, "loader shapes");
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave >> 1, wave_n = wave & 1;
  const int l31 = lane & 31, lhalf = lane >> 5;

  const int s = a.dw_stride;
  const int PH = (a.th - 1) * s + 3, PWd = (a.tw - 1) * s + 3;      // staged block of the pointwise output
  unsigned char* s_mid = smem;
  unsigned char* s_op = smem + PH * PWd * MP;
  const int nsteps = a.Kred_pad / BKE;
  const int tiles_sp = a.tiles_y * a.tiles_x;
  const int cg = tid % CG;

  for (int t = blockIdx.x; t < a.ntiles; t += gridDim.x) {
    const int tile_n = t / a.tiles_m, tm = t - tile_n * a.tiles_m;  // neighbours share a weight slice
    const int n = tm / tiles_sp, rr = tm - n * tiles_sp, ty = rr / a.tiles_x, tx = rr - ty * a.tiles_x;
    const int oy0 = ty * a.th, ox0 = tx * a.tw;                    // first depthwise output pixel of the tile
    const int iy0 = oy0 * s - 1, ix0 = ox0 * s - 1;                // map position of block position (0, 0)
    const int y_lo = iy0 > 0 ? iy0 : 0, y_hi = iy0 + PH < a.H ? iy0 + PH : a.H;
    const int x_lo = ix0 > 0 ? ix0 : 0, x_hi = ix0 + PWd < a.W ? ix0 + PWd : a.W;
    const int hv = y_hi - y_lo, wv = x_hi - x_lo, npos = hv * wv;   // the part of the block inside the map (never empty)

    // this thread's depthwise weights and folded scale / shift: its channel group is the same for all its pixels
    const int k0 = tile_n * BN + cg * CE;
    const bool kok = k0 < a.K;
    u32x4_t dww[9];
#pragma unroll
    for (int t9 = 0; t9 < 9; ++t9) dww[t9] = *(const u32x4_t*)((const T*)a.dw_w + (long long)t9 * a.K + (kok ? k0 : 0));

    if (hv < PH || wv < PWd) {
      // the block overhangs the map: those positions are the zero padding of the depthwise convolution
      const u32x4_t z = {0u, 0u, 0u, 0u};
      for (int i = tid; i < PH * PWd * (MP / 16); i += NT) *(u32x4_t*)(s_mid + i * 16) = z;
    }

    for (int mc = 0; mc * BM < npos; ++mc) {
      // ---- pointwise GEMM of 64 block positions x 64 channels over all input channels ----------------
      long long abase[A_IT];
      bool arow[A_IT];
      const int ch = tid % CPR;
#pragma unroll
      for (int it = 0; it < A_IT; ++it) {
        const int m = mc * BM + (tid + it * NT) / CPR;
        arow[it] = m < npos;
        const int mm = arow[it] ? m : 0;
        const int py = mm / wv, px = mm - py * wv;
        abase[it] = (long long)n * a.in_sN + (long long)(y_lo + py) * a.in_sH + (long long)(x_lo + px) * a.in_sW + ch * CE;
      }
      const unsigned char* wrow[B_IT];
#pragma unroll
      for (int it = 0; it < B_IT; ++it) {
        const int idx = tid + it * NT;
        wrow[it] = (const unsigned char*)a.w + ((long long)(tile_n * BN + idx / CPR) * a.Kred_pad + (idx % CPR) * CE) * (long long)ESZ;
      }
      f32x16_t acc;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = 0.f;
      u32x4_t ra0[A_IT], rb0[B_IT], ra1[A_IT], rb1[B_IT];
      auto load = [&](int step, u32x4_t* ra, u32x4_t* rb) {
        const int ss = step < nsteps ? step : nsteps - 1;          // steps past the end re-read valid memory; never used
        const int kc = ss * BKE + ch * CE;
        const u32x4_t z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int it = 0; it < A_IT; ++it) {
          const bool ok = arow[it] && kc < a.C;                    // channels beyond C are the padding of the reduction
          const u32x4_t v = *(const u32x4_t*)((const T*)a.in + (ok ? abase[it] + ss * BKE : 0));
          ra[it] = ok ? v : z;
        }
#pragma unroll
        for (int it = 0; it < B_IT; ++it) rb[it] = *(const u32x4_t*)(wrow[it] + (long long)ss * ROWB);
      };
      auto store = [&](int stage, const u32x4_t* ra, const u32x4_t* rb) {
        unsigned char* sa = s_op + stage * (BM + BN) * LDS_ROW;
        unsigned char* sb = sa + BM * LDS_ROW;
#pragma unroll
        for (int it = 0; it < A_IT; ++it) {
          const int idx = tid + it * NT;
          *(u32x4_t*)(sa + (idx / CPR) * LDS_ROW + (idx % CPR) * 16) = ra[it];
        }
#pragma unroll
        for (int it = 0; it < B_IT; ++it) {
          const int idx = tid + it * NT;
          *(u32x4_t*)(sb + (idx / CPR) * LDS_ROW + (idx % CPR) * 16) = rb[it];
        }
      };
      auto compute = [&](int stage) {
        const unsigned char* sa = s_op + stage * (BM + BN) * LDS_ROW + (wave_m * 32 + l31) * LDS_ROW + lhalf * 16;
        const unsigned char* sb = s_op + stage * (BM + BN) * LDS_ROW + BM * LDS_ROW + (wave_n * 32 + l31) * LDS_ROW + lhalf * 16;
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
      load(0, ra0, rb0);
      store(0, ra0, rb0);
      load(1, ra1, rb1);
      __syncthreads();                                             // step 0 (and the zero fill of the block) is visible
      for (int st = 0; st < nsteps; st += 2) {
        load(st + 2, ra0, rb0);
        compute(0);
        store(1, ra1, rb1);
        __syncthreads();
        if (st + 1 >= nsteps) break;
        load(st + 3, ra1, rb1);
        compute(1);
        store(0, ra0, rb0);
        __syncthreads();
      }
      // ---- the pointwise chain's epilogue, into the LDS block: lane = position wave_m*32 + l31, channels
      // wave_n*32 + 8*g + 4*lhalf + (0..3) ------------------------------------------------------------
      const int m = mc * BM + wave_m * 32 + l31;
      if (m < npos) {
        const int py = m / wv, px = m - py * wv;
        unsigned char* dst = s_mid + ((y_lo + py - iy0) * PWd + (x_lo + px - ix0)) * MP;
        const float lo = a.relu ? 0.f : -3.4028235e38f;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int c = wave_n * 32 + g * 8 + lhalf * 4, kk = tile_n * BN + c;
          const f32x4_t sc = *(const f32x4_t*)(a.scale + kk), sh = *(const f32x4_t*)(a.shift + kk);
          float y[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) y[e] = fmx(acc[4 * g + e] * sc[e] + sh[e], lo);
          if constexpr (sizeof(T) == 2) {
            uint2 o;
            o.x = f2bf2(y[0], y[1]);
            o.y = f2bf2(y[2], y[3]);
            *(uint2*)(dst + c * 2) = o;
          } else {
            *(f32x4_t*)(dst + c * 4) = f32x4_t{y[0], y[1], y[2], y[3]};
          }
        }
      }
    }
    __syncthreads();                                               // the block is complete

    // ---- depthwise chain out of the block: one thread = one 16-byte channel group of one output pixel --------
    if (kok) {
      float dsc[CE], dsh[CE];
#pragma unroll
      for (int e = 0; e < CE; e += 4) {
        *(f32x4_t*)&dsc[e] = *(const f32x4_t*)(a.dw_scale + k0 + e);
        *(f32x4_t*)&dsh[e] = *(const f32x4_t*)(a.dw_shift + k0 + e);
      }
      for (int q = tid / CG; q < a.th * a.tw; q += NT / CG) {
        const int qy = q / a.tw, qx = q - qy * a.tw;
        const int oy = oy0 + qy, ox = ox0 + qx;
        if (oy >= a.OH || ox >= a.OW) continue;
        const unsigned char* src = s_mid + ((qy * s) * PWd + qx * s) * MP + cg * 16;
        float d[CE];
#pragma unroll
        for (int e = 0; e < CE; ++e) d[e] = 0.f;
#pragma unroll
        for (int t9 = 0; t9 < 9; ++t9) {
          float x[CE], w[CE];
          tr::unpack(*(const u32x4_t*)(src + ((t9 / 3) * PWd + t9 % 3) * MP), x);
          tr::unpack(dww[t9], w);
#pragma unroll
          for (int e = 0; e < CE; ++e) d[e] = fmaf(x[e], w[e], d[e]);
        }
#pragma unroll
        for (int e = 0; e < CE; ++e) {
          const float y = d[e] * dsc[e] + dsh[e];
          d[e] = a.dw_relu ? fmx(y, 0.f) : y;
        }
        *(u32x4_t*)((T*)a.out + (long long)n * a.out_sN + (long long)(oy * a.OW + ox) * a.out_sP + k0) = tr::pack(d);
      }
    }
    __syncthreads();                                               // the block is rewritten by the next tile
  }
}

template <typename T>
static int launch_pwdw_t(const ConvArgs& a, hipStream_t st) {
  constexpr int ESZ = (int)sizeof(T), BKE = Tr<T>::BKE, CE = Tr<T>::CE;
  const int s = a.dw_stride;
  // what the kernel assumes, checked again on the host: a wrong shape would index outside the LDS block or the tensors
  if (a.mode != M_FLAT || a.has_res || a.pool != POOL_NONE || a.ksplit >= 1 || a.ileave || a.kchunk || a.pair || a.dw_panel ||
      a.R != 1 || a.S != 1 || a.stride != 1 || a.pad != 0 || a.C % CE != 0 || a.K % CE != 0 || a.C < CE ||
      a.Kred_pad < (a.C + BKE - 1) / BKE * BKE || a.Kred_pad % BKE != 0 ||
      a.dw_k != 3 || a.dw_pad != 1 || (s != 1 && s != 2) || !a.dw_w || !a.dw_scale || !a.dw_shift || !a.vec_out ||
      a.OH != (a.H + 2 - 3) / s + 1 || a.OW != (a.W + 2 - 3) / s + 1 || a.th < 1 || a.tw < 1 ||
      a.tiles_y != (a.OH + a.th - 1) / a.th || a.tiles_x != (a.OW + a.tw - 1) / a.tw || a.tiles_m != a.N * a.tiles_y * a.tiles_x ||
      a.tiles_n != (a.K + PD_BN - 1) / PD_BN || a.ntiles != a.tiles_m * a.tiles_n || a.grid < 1 ||
      a.in_sN < 0 || a.in_sH < 0 || a.in_sW < a.C || a.out_sP < a.K)
    return (int)hipErrorInvalidValue;
  const int positions = ((a.th - 1) * s + 3) * ((a.tw - 1) * s + 3);
  const int lds = pwdw_lds(positions, ESZ);
  if (positions > kPwDwMaxPositions || lds > 160 * 1024) return (int)hipErrorInvalidValue;
  static int raised = 0;
  if (lds > raised) {
    hipError_t e = hipFuncSetAttribute((const void*)pwdw_kernel<T>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return (int)e;
    raised = lds;
  }
  hipLaunchKernelGGL((pwdw_kernel<T>), dim3(a.grid < a.ntiles ? a.grid : a.ntiles), dim3(NT), lds, st, a);
  return (int)hipGetLastError();
}

int launch_pwdw(const ConvArgs& a, int dtype, void* stream) {
  return dtype == DT_BF16 ? launch_pwdw_t<bf16_t>(a, (hipStream_t)stream) : launch_pwdw_t<float>(a, (hipStream_t)stream);
}

size_t pwdw_lds_bytes(int th, int tw, int stride, int esz) {
  return (size_t)pwdw_lds(((th - 1) * stride + 3) * ((tw - 1) * stride + 3), esz);
}

}  // namespace xenos
