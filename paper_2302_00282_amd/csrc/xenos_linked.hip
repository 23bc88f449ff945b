// gfx950 (CDNA4) kernels of the chains whose intermediate tensor stays on chip between two convolutions
// (Table 1, ConvX -> ConvY; Section 2.2 and the last paragraph of Section 4.1):
//
//  pwdw_kernel   pointwise (1x1) convolution chain -> depthwise 3x3 convolution chain.  The pointwise output of a
//                spatial tile plus the one-pixel halo the depthwise windows need lives in LDS only, written there by
//                the GEMM epilogue in the [position][channel] order the depthwise stencil reads.
//  fire_kernel   squeeze 1x1 -> { expand 1x1 || expand 3x3 } -> concat [-> max-pooling] (a Fire module) as one chain: the
//                squeeze tile (+ halo) lives in LDS and is the pixel operand of both expand GEMMs.
#include "device_common.h"

namespace xenos {

// ---------------------------------------------------------------------------------------------
// The 1x1 / stride 1 convolution over all a.C input channels that both kernels below start with, in chunks of 64 pixels x
// 64 output channels.  4 wavefronts as 2 x 2 of 32 pixels x 32 channels; the GEMM is computed transposed, so a lane of
// wavefront (wave_m, wave_n) holds, for pixel row wave_m*32 + l%32, channels k_row0 + wave_n*32 + 8*g + 4*(l/32) + (0..3)
// in acc[4*g .. 4*g+3].  Two LDS stages at s_op (2 * (64 + 64) * LDS_ROW bytes).
// ---------------------------------------------------------------------------------------------
constexpr int PG_BM = 64, PG_BN = 64;
constexpr int PG_STAGES_BYTES = 2 * (PG_BM + PG_BN) * LDS_ROW;

// The GEMMs of ALL chunks of a phase as one sequence of steps (chunk 0 step 0, step 1, ..., chunk 1 step 0, ...): the
// operands of step g + PG_DEPTH are requested from memory when step g is staged, so the memory latency (about 1 us at
// batch 32; timestamps inside the kernels showed it exposed once per chunk, 1.4 us per chunk of a 64-channel layer of
// which 0.3 are work) passes behind the steps before it, across chunk boundaries too.  A ring of PG_DEPTH register sets
// holds the requests in flight, two LDS stages hold the step being multiplied and the next one, one barrier per step.
// pixel(chunk, row) gives the element offset of a row's input pixel (-1 = no pixel); epilogue(chunk, acc) receives
// the finished accumulators of a chunk (lane = row wave_m * 32 + l31, channels wave_n * 32 + 8 g + 4 lhalf + 0..3).
// Ends without a barrier: the caller's next barrier frees the stages.
// TAPS = 9: the convolution is 3x3 / stride 1 / pad 1 instead of 1x1, its weights packed with all taps of a chunk of BKE
// channels in consecutive steps (a.C a multiple of BKE): step s is tap s % 9 of chunk s / 9, the input element of a row
// is its pixel's neighbour at that tap, zero outside the map; coord(chunk, row) gives the pixel's (y << 16) | x.
constexpr int PG_DEPTH = 4;

struct NoCoord { __device__ __forceinline__ int operator()(int, int) const { return 0; } };

template <typename T, int TAPS = 1, typename PixelFn, typename EpiFn, typename CoordFn = NoCoord>
__device__ __forceinline__ void pw_gemm_phase(const ConvArgs& a, int k_row0, unsigned char* s_op, int nchunks, PixelFn pixel, EpiFn epilogue,
                                              CoordFn coord = CoordFn()) {
  static_assert(TAPS == 1 || TAPS == 9, "1x1 or 3x3 / pad 1");
  using tr = Tr<T>;
  constexpr int CE = tr::CE, BKE = tr::BKE, ESZ = (int)sizeof(T);
  constexpr int BM = PG_BM, BN = PG_BN, D = PG_DEPTH;
  constexpr int A_IT = BM * CPR / NT, B_IT = BN * CPR / NT;        // 16-byte chunks per thread and step
  static_assert(A_IT >= 1 && B_IT >= 1 && A_IT <= 8 && D % 2 == 0, "loader shapes");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave >> 1, wave_n = wave & 1;
  const int l31 = lane & 31, lhalf = lane >> 5;
  const int nsteps = a.Kred_pad / BKE, G = nchunks * nsteps;
  const int ch = tid % CPR;
  const unsigned char* wrow[B_IT];
#pragma unroll
  for (int it = 0; it < B_IT; ++it) {
    const int idx = tid + it * NT;
    wrow[it] = (const unsigned char*)a.w + ((long long)(k_row0 + idx / CPR) * a.Kred_pad + (idx % CPR) * CE) * (long long)ESZ;
  }
  // the chunk and step the next request belongs to, and this thread's input rows of that chunk
  int ld_chunk = -1, ld_step = nsteps - 1;
  long long abase[A_IT];
  int ayx[TAPS == 9 ? A_IT : 1];                                   // TAPS = 9: (y << 16) | x of this thread's rows
  unsigned arow = 0;
  u32x4_t ra[D][A_IT], rb[D][B_IT];
  unsigned okm[D];                                                 // which of a set's input chunks are real (the others are zero)
  auto request = [&](int q, int d) __attribute__((always_inline)) {
    if (q >= G) return;                                            // (uniform)
    if (++ld_step == nsteps) {
      ld_step = 0;
      ++ld_chunk;
      arow = 0;
#pragma unroll
      for (int it = 0; it < A_IT; ++it) {
        const long long off = pixel(ld_chunk, (tid + it * NT) / CPR);
        arow |= (off >= 0 ? 1u : 0u) << it;
        abase[it] = (off >= 0 ? off : 0) + ch * CE;
        if constexpr (TAPS == 9) ayx[it] = coord(ld_chunk, (tid + it * NT) / CPR);
      }
    }
    if constexpr (TAPS == 9) {
      const int cch = ld_step / 9, tap = ld_step - cch * 9, dy = tap / 3 - 1, dx = tap - (tap / 3) * 3 - 1;
      const long long toff = (long long)dy * a.in_sH + (long long)dx * a.in_sW + (long long)cch * BKE;
      unsigned ok = 0;
#pragma unroll
      for (int it = 0; it < A_IT; ++it) {
        const int y = (ayx[it] >> 16) + dy, x = (ayx[it] & 0xffff) + dx;
        ok |= (((arow >> it) & 1u) && (unsigned)y < (unsigned)a.H && (unsigned)x < (unsigned)a.W ? 1u : 0u) << it;
      }
      okm[d] = ok;
#pragma unroll
      for (int it = 0; it < A_IT; ++it)
        ra[d][it] = *(const u32x4_t*)((const T*)a.in + (((ok >> it) & 1u) ? abase[it] + toff : 0));
    } else {
      const int kc = ld_step * BKE + ch * CE;
      okm[d] = kc < a.C ? arow : 0u;                               // channels beyond C are the padding of the reduction
#pragma unroll
      for (int it = 0; it < A_IT; ++it)
        ra[d][it] = *(const u32x4_t*)((const T*)a.in + (((okm[d] >> it) & 1u) ? abase[it] + ld_step * BKE : 0));
    }
#pragma unroll
    for (int it = 0; it < B_IT; ++it) rb[d][it] = *(const u32x4_t*)(wrow[it] + (long long)ld_step * ROWB);
  };
  auto store = [&](int stage, int d) __attribute__((always_inline)) {
    unsigned char* sa = s_op + stage * (BM + BN) * LDS_ROW;
    unsigned char* sb = sa + BM * LDS_ROW;
    const u32x4_t z = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
      const int idx = tid + it * NT;
      *(u32x4_t*)(sa + (idx / CPR) * LDS_ROW + (idx % CPR) * 16) = ((okm[d] >> it) & 1u) ? ra[d][it] : z;
    }
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
      const int idx = tid + it * NT;
      *(u32x4_t*)(sb + (idx / CPR) * LDS_ROW + (idx % CPR) * 16) = rb[d][it];
    }
  };
  f32x16_t acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  auto compute = [&](int stage) __attribute__((always_inline)) {
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
#pragma unroll
  for (int d = 0; d < D; ++d) request(d, d);
  int c_chunk = 0, c_step = 0;
  for (int g0 = 0; g0 < G; g0 += D) {
#pragma unroll
    for (int d = 0; d < D; ++d) {
      const int g = g0 + d;
      if (g < G) {                                                 // (uniform)
        // stage d % 2 was last read by step g - 2, which every wavefront finished before the barrier of step g - 1
        store(d & 1, d);
        request(g + D, d);
        __syncthreads();                                           // step g (and whatever the caller wrote before the phase) is visible
        compute(d & 1);
        if (++c_step == nsteps) {
          epilogue(c_chunk, acc);
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[e] = 0.f;
          c_step = 0;
          ++c_chunk;
        }
      }
    }
  }
}

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
  static_assert(NT % CG == 0 && BM == PG_BM && BN == PG_BN, "loader shapes");
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave >> 1, wave_n = wave & 1;
  const int l31 = lane & 31, lhalf = lane >> 5;

  const int s = a.dw_stride;
  const int PH = (a.th - 1) * s + 3, PWd = (a.tw - 1) * s + 3;      // staged block of the pointwise output
  unsigned char* s_mid = smem;
  unsigned char* s_op = smem + PH * PWd * MP;
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

    // scale and shift of this lane's channels: the same for every chunk, requested once
    f32x4_t psc[4], psh[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int kk = tile_n * BN + wave_n * 32 + g * 8 + lhalf * 4;
      psc[g] = *(const f32x4_t*)(a.scale + kk);
      psh[g] = *(const f32x4_t*)(a.shift + kk);
    }
    // ---- pointwise GEMM of the block, 64 positions x 64 channels per chunk over all input channels, and the pointwise
    // chain's epilogue into the LDS block: lane = position wave_m*32 + l31, channels wave_n*32 + 8*g + 4*lhalf + (0..3)
    pw_gemm_phase<T>(a, tile_n * BN, s_op, (npos + BM - 1) / BM, [&](int mc, int row) -> long long {
      const int m = mc * BM + row;
      if (m >= npos) return -1;
      const int py = m / wv, px = m - py * wv;
      return (long long)n * a.in_sN + (long long)(y_lo + py) * a.in_sH + (long long)(x_lo + px) * a.in_sW;
    }, [&](int mc, const f32x16_t& acc) {
      const int m = mc * BM + wave_m * 32 + l31;
      if (m < npos) {
        const int py = m / wv, px = m - py * wv;
        unsigned char* dst = s_mid + ((y_lo + py - iy0) * PWd + (x_lo + px - ix0)) * MP;
        const float lo = a.relu ? 0.f : -3.4028235e38f;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int c = wave_n * 32 + g * 8 + lhalf * 4;
          const f32x4_t sc = psc[g], sh = psh[g];
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
    });
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

// ---------------------------------------------------------------------------------------------
// Fire module on chip: squeeze 1x1 -> { expand 1x1  ||  expand 3x3 / pad 1 } -> channel concat [-> max-pooling] as ONE
// chain (Table 1, Conv1x1 -> Conv3x3; Section 4.1, last paragraph: the consumer's halo is replicated per tile).
//
// The squeeze output has few channels (16 .. 64) and two readers; kept in LDS it is written once and never reaches
// memory.  A workgroup owns a TH x TW tile of output pixels of one image and a share of the expand channels:
//   phase 1  the squeeze chain (GEMM over all input channels + scale/shift + ReLU) for the (TH+2) x (TW+2) block of
//            pixels the 3x3 windows cover, in chunks of 64 positions, into an LDS block [position][S channels] in the
//            storage type; positions outside the map stay zero (the padding of the 3x3 convolution);
//   phase 2  for each of its 64-channel expand tiles: the tile's weights (all taps) are copied to LDS once, then every
//            chunk of 64 pixels runs its 1 or 9 taps as MFMAs whose pixel operand is read from the squeeze block at the
//            tap's offset and whose weight operand from the resident tile: no barrier inside; the epilogue (scale/shift/
//            ReLU) is per wavefront, staged through a private LDS slice and stored as 16-byte channel groups at the
//            part's channel offset in the concat buffer (Eq. 1: the halves join without a layout pass).
// With a linked 3x3 / stride 2 max-pooling (ceil mode; the planner hoists the pooling over the concat) the tile is PTH x
// PTW pooling windows: the expand results of the (2 PTH + 1) x (2 PTW + 1) pixels they cover are staged per channel tile
// in LDS and one thread per 16-byte channel group of a window takes the maximum.
// Workgroups of different channel shares recompute the squeeze block of their tile.
// ---------------------------------------------------------------------------------------------
__host__ __device__ constexpr int fire_sq_pitch(int S, int esz) { return S * esz + 16; }
__host__ __device__ constexpr int fire_w_pitch(int taps, int S, int esz) { return taps * S * esz + 16; }
__host__ __device__ constexpr int fire_stg_pitch(int esz) { return 32 * esz + 16; }
__host__ __device__ constexpr int fire_cb_pitch(int esz) { return 64 * esz + 16; }
// LDS: squeeze block | max(GEMM stages, one 3x3 weight tile) | 4 per-wavefront staging slices | pooled form: conv block of a channel tile
__host__ __device__ constexpr int fire_lds(int positions, int S, int esz, int pool_positions) {
  return positions * fire_sq_pitch(S, esz) + cmax(PG_STAGES_BYTES, 64 * fire_w_pitch(9, S, esz)) + 4 * 32 * fire_stg_pitch(esz) +
         pool_positions * fire_cb_pitch(esz);
}

template <typename T, bool POOL, int TAPS1>
__global__ __launch_bounds__(NT) void fire_kernel(const ConvArgs a) {
  using tr = Tr<T>;
  constexpr int CE = tr::CE, ESZ = (int)sizeof(T);
  constexpr int STP = fire_stg_pitch(ESZ), CBP = fire_cb_pitch(ESZ);
  constexpr int G = 32 * ESZ / 16;                                 // 16-byte channel groups of a wavefront's 32 channels
  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wave_m = wave >> 1, wave_n = wave & 1;
  const int l31 = lane & 31, lhalf = lane >> 5;

  const int S = a.K;                                               // squeeze channels
  const int SQP = fire_sq_pitch(S, ESZ);
  const int kgs = S * ESZ / 32;                                    // MFMA k-groups per tap
  // conv-output pixels of a tile: th x tw, or the block the tile's pooling windows cover
  const int CH = POOL ? (a.pph - 1) * a.ps + a.pk : a.th, CW = POOL ? (a.ppw - 1) * a.ps + a.pk : a.tw;
  // the block of the first convolution's output a tile reads: its pixels, and one ring of halo when a 3x3 part exists
  const int ring = a.fire_E[1] > 0 ? 1 : 0;
  const int PH = CH + 2 * ring, PWd = CW + 2 * ring;
  unsigned char* s_sq = smem;
  unsigned char* s_b = smem + PH * PWd * SQP;
  const int bbytes = 64 * fire_w_pitch(9, S, ESZ);
  unsigned char* s_stg = s_b + (bbytes > PG_STAGES_BYTES ? bbytes : PG_STAGES_BYTES) + wave * 32 * STP;
  unsigned char* s_cb = s_b + (bbytes > PG_STAGES_BYTES ? bbytes : PG_STAGES_BYTES) + 4 * 32 * STP;   // POOL: [conv pixel][64 channels]
  const int tiles_sp = a.tiles_y * a.tiles_x;
  const int npix = CH * CW;

  for (int t = blockIdx.x; t < a.ntiles; t += gridDim.x) {
    const int gz = t / a.tiles_m, tm = t - gz * a.tiles_m;          // channel share, spatial tile
    const int n = tm / tiles_sp, rr = tm - n * tiles_sp, ty = rr / a.tiles_x, tx = rr - ty * a.tiles_x;
    // first conv-output pixel of the tile
    const int oy0 = POOL ? ty * a.pph * a.ps - a.pp : ty * a.th, ox0 = POOL ? tx * a.ppw * a.ps - a.pp : tx * a.tw;
    const int iy0 = oy0 - ring, ix0 = ox0 - ring;                  // map position of block position (0, 0)
    const int y_lo = iy0 > 0 ? iy0 : 0, y_hi = iy0 + PH < a.H ? iy0 + PH : a.H;
    const int x_lo = ix0 > 0 ? ix0 : 0, x_hi = ix0 + PWd < a.W ? ix0 + PWd : a.W;
    const int hv = y_hi - y_lo, wv = x_hi - x_lo, npos = hv * wv;   // the part of the block inside the map (never empty)

    if (hv < PH || wv < PWd) {
      const u32x4_t z = {0u, 0u, 0u, 0u};
      for (int i = tid; i < PH * PWd * (SQP / 16); i += NT) *(u32x4_t*)(s_sq + i * 16) = z;
    }
    // ---- phase 1: the squeeze chain of the block, into LDS -------------------------------------------------
    // (scale and shift of this lane's channels are the same for every chunk: requested once)
    f32x4_t qsc[4], qsh[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const int c = wave_n * 32 + g * 8 + lhalf * 4;
      qsc[g] = *(const f32x4_t*)(a.scale + (c < S ? c : 0));
      qsh[g] = *(const f32x4_t*)(a.shift + (c < S ? c : 0));
    }
    pw_gemm_phase<T, TAPS1>(a, 0, s_b, (npos + 63) / 64, [&](int mc, int row) -> long long {
      const int m = mc * 64 + row;
      if (m >= npos) return -1;
      const int py = m / wv, px = m - py * wv;
      return (long long)n * a.in_sN + (long long)(y_lo + py) * a.in_sH + (long long)(x_lo + px) * a.in_sW;
    }, [&](int mc, const f32x16_t& acc) {
      const int m = mc * 64 + wave_m * 32 + l31;
      if (m < npos) {
        const int py = m / wv, px = m - py * wv;
        unsigned char* dst = s_sq + ((y_lo + py - iy0) * PWd + (x_lo + px - ix0)) * SQP;
        const float lo = a.relu ? 0.f : -3.4028235e38f;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int c = wave_n * 32 + g * 8 + lhalf * 4;
          if (c < S) {
            const f32x4_t sc = qsc[g], sh = qsh[g];
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
    }, [&](int mc, int row) -> int {
      const int m = mc * 64 + row, mm = m < npos ? m : 0;
      const int py = mm / wv, px = mm - py * wv;
      return ((y_lo + py) << 16) | (x_lo + px);
    });
    __syncthreads();                                               // the block is complete, the GEMM stages are free

    // ---- phase 2: this workgroup's expand tiles -----------------------------------------------------------
#pragma unroll 1
    for (int which = 0; which < 2; ++which) {                      // 0: the 1x1 expand, 1: the 3x3 expand
      const int taps = which ? 9 : 1, E = a.fire_E[which];
      const int WP = fire_w_pitch(taps, S, ESZ), wrow_b = taps * S * ESZ;   // LDS pitch and bytes of a channel's weights
      const float lo = a.fire_relu[which] ? 0.f : -3.4028235e38f;
#pragma unroll 1
      for (int j = gz; j * 64 < E; j += a.tiles_n) {
        {   // the tile's weights: 64 channels x taps x S, contiguous in memory (rows beyond E are zero)
          const unsigned char* src = (const unsigned char*)a.fire_w[which] + (long long)j * 64 * wrow_b;
          const int cpr = wrow_b / 16, total = 64 * cpr;
          // six requests per thread before the first is written to LDS: as a loop of load-then-store the copy paid one
          // memory latency per 4 KB (timestamps inside the kernel: 3.2 us for the 72 KB of a 3x3 tile over 64 channels)
          constexpr int CB = 6;
          for (int idx0 = tid; idx0 < total; idx0 += CB * NT) {
            u32x4_t wv[CB];
#pragma unroll
            for (int u = 0; u < CB; ++u) {
              const int idx = idx0 + u * NT;
              wv[u] = *(const u32x4_t*)(src + (long long)(idx < total ? idx : 0) * 16);   // (the tile is contiguous in memory)
            }
#pragma unroll
            for (int u = 0; u < CB; ++u) {
              const int idx = idx0 + u * NT, row = idx / cpr, c = idx - row * cpr;
              if (idx < total) *(u32x4_t*)(s_b + row * WP + c * 16) = wv[u];
            }
          }
        }
        __syncthreads();
#pragma unroll 1
        for (int mc = 0; mc * 64 < npix; ++mc) {
          const int m = mc * 64 + wave_m * 32 + l31;
          const int mm = m < npix ? m : 0;
          const int py = mm / CW, px = mm - py * CW;
          // block position of the pixel's first tap: the 1x1 expand reads the pixel itself, the 3x3 its window
          const unsigned char* pa = s_sq + ((py + (which ? 0 : ring)) * PWd + px + (which ? 0 : ring)) * SQP + lhalf * 16;
          const unsigned char* pb = s_b + (wave_n * 32 + l31) * WP + lhalf * 16;
          f32x16_t acc;
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll 1
          for (int tap = 0; tap < taps; ++tap) {
            const unsigned char* ta = pa + ((tap / 3) * PWd + tap % 3) * SQP;
            const unsigned char* tb = pb + tap * S * ESZ;
            for (int kg = 0; kg < kgs; ++kg) {
              const u32x4_t fa = *(const u32x4_t*)(ta + kg * 32), fb = *(const u32x4_t*)(tb + kg * 32);
              if constexpr (sizeof(T) == 2) {
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fb), __builtin_bit_cast(bf16x8_t, fa), acc, 0, 0, 0);
              } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                  acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fb[e]), __uint_as_float(fa[e]), acc, 0, 0, 0);
              }
            }
          }
          // epilogue of the wavefront's 32 pixels x 32 channels: finished values change hands inside the wavefront only
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const int c = g * 8 + lhalf * 4, kk = j * 64 + wave_n * 32 + c;
            const f32x4_t sc = *(const f32x4_t*)(a.fire_scale[which] + kk), sh = *(const f32x4_t*)(a.fire_shift[which] + kk);
            float y[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) y[e] = fmx(acc[4 * g + e] * sc[e] + sh[e], lo);
            if constexpr (sizeof(T) == 2) {
              uint2 o;
              o.x = f2bf2(y[0], y[1]);
              o.y = f2bf2(y[2], y[3]);
              *(uint2*)(s_stg + l31 * STP + c * 2) = o;
            } else {
              *(u32x4_t*)(s_stg + l31 * STP + c * 4) = u32x4_t{__float_as_uint(y[0]), __float_as_uint(y[1]), __float_as_uint(y[2]), __float_as_uint(y[3])};
            }
          }
#pragma unroll
          for (int u = 0; u < 32 * G / 64; ++u) {
            const int idx = lane + u * 64, r = idx / G, cg = idx - r * G;
            const int mr = mc * 64 + wave_m * 32 + r;
            const int k0 = j * 64 + wave_n * 32 + cg * CE;
            u32x4_t v;
            if constexpr (sizeof(T) == 2) {
              const uint2 lo8 = *(const uint2*)(s_stg + r * STP + cg * 16), hi8 = *(const uint2*)(s_stg + r * STP + cg * 16 + 8);
              v = u32x4_t{lo8.x, lo8.y, hi8.x, hi8.y};
            } else {
              v = *(const u32x4_t*)(s_stg + r * STP + cg * 16);
            }
            if (mr < npix && k0 < E) {
              const int qy = mr / CW, qx = mr - qy * CW;
              if constexpr (POOL) {
                *(u32x4_t*)(s_cb + mr * CBP + (wave_n * 32 + cg * CE) * ESZ) = v;
              } else {
                const int oy = oy0 + qy, ox = ox0 + qx;
                if (oy < a.H && ox < a.W)
                  *(u32x4_t*)((T*)a.fire_out[which] + (long long)n * a.fire_sN[which] + (long long)(oy * a.W + ox) * a.fire_sP[which] + k0) = v;
              }
            }
          }
        }
        if constexpr (POOL) {
          __syncthreads();                                         // the conv block of this channel tile is complete
          // one thread = one 16-byte channel group of one pooling window; windows are clipped to the map (never empty)
          constexpr int CG = 64 / CE;
          for (int idx = tid; idx < a.pph * a.ppw * CG; idx += NT) {
            const int q = idx / CG, cg = idx - q * CG, k0 = j * 64 + cg * CE;
            const int qy = q / a.ppw, qx = q - qy * a.ppw;
            const int gy = ty * a.pph + qy, gx = tx * a.ppw + qx;
            if (gy >= a.PH || gx >= a.PW || k0 >= E) continue;
            float mx[CE];
#pragma unroll
            for (int e = 0; e < CE; ++e) mx[e] = -INFINITY;
            if (a.pk == 3) {
              // all nine reads of the window are issued before the first maximum (elements outside the map read the
              // window's first element, which is inside, once more): as a loop over rows and columns the stage paid one
              // LDS latency per element, 3 of the 21 us of a pooled module's workgroup at batch 32
              u32x4_t wv9[9];
#pragma unroll
              for (int t9 = 0; t9 < 9; ++t9) {
                const int cy = qy * a.ps + t9 / 3, cx = qx * a.ps + t9 % 3;
                const bool in = oy0 + cy < a.H && ox0 + cx < a.W;   // (no padding: windows start inside the map)
                wv9[t9] = *(const u32x4_t*)(s_cb + (in ? cy * CW + cx : qy * a.ps * CW + qx * a.ps) * CBP + cg * 16);
              }
#pragma unroll
              for (int t9 = 0; t9 < 9; ++t9) {
                float x[CE];
                tr::unpack(wv9[t9], x);
#pragma unroll
                for (int e = 0; e < CE; ++e) mx[e] = fmx_raw(mx[e], x[e]);
              }
            } else {
              for (int r = 0; r < a.pk; ++r)
                for (int c = 0; c < a.pk; ++c) {
                  const int cy = qy * a.ps + r, cx = qx * a.ps + c;
                  const int oy = oy0 + cy, ox = ox0 + cx;
                  if (oy < 0 || oy >= a.H || ox < 0 || ox >= a.W) continue;
                  float x[CE];
                  tr::unpack(*(const u32x4_t*)(s_cb + (cy * CW + cx) * CBP + cg * 16), x);
#pragma unroll
                  for (int e = 0; e < CE; ++e) mx[e] = fmx_raw(mx[e], x[e]);
                }
            }
            *(u32x4_t*)((T*)a.fire_out[which] + (long long)n * a.fire_sN[which] + (long long)(gy * a.PW + gx) * a.fire_sP[which] + k0) = tr::pack(mx);
          }
        }
        __syncthreads();                                           // the weight tile (and the conv block) are rewritten
      }
    }
  }
}

template <typename T, bool POOL, int TAPS1>
static int launch_fire_inst(const ConvArgs& a, int lds, hipStream_t st) {
  static int raised = 0;
  if (lds > raised) {
    hipError_t e = hipFuncSetAttribute((const void*)fire_kernel<T, POOL, TAPS1>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return (int)e;
    raised = lds;
  }
  hipLaunchKernelGGL((fire_kernel<T, POOL, TAPS1>), dim3(a.grid < a.ntiles ? a.grid : a.ntiles), dim3(NT), lds, st, a);
  return (int)hipGetLastError();
}

template <typename T>
static int launch_fire_t(const ConvArgs& a, hipStream_t st) {
  constexpr int ESZ = (int)sizeof(T), BKE = Tr<T>::BKE, CE = Tr<T>::CE;
  const bool pool = a.pool != POOL_NONE;
  // what the kernel assumes, checked again on the host
  // the first convolution: 1x1 / pad 0, or 3x3 / pad 1 with the taps of a channel chunk packed in consecutive steps
  const bool first3 = a.R == 3;
  if (a.mode != M_FLAT || a.has_res || a.ksplit >= 1 || a.ileave || a.pair || a.dw_panel || a.pwdw || a.dw_w || a.stride != 1 || a.R != a.S ||
      (first3 ? (a.pad != 1 || !a.kchunk || a.C % BKE != 0 || a.Kred_pad != 9 * a.C || a.H > 0xffff || a.W > 0xffff)
              : (a.R != 1 || a.pad != 0 || a.kchunk || a.Kred_pad < (a.C + BKE - 1) / BKE * BKE)) ||
      a.C % CE != 0 || a.C < CE || a.Kred_pad % BKE != 0 ||
      a.K < 1 || a.K > 64 || (a.K * ESZ) % 32 != 0 || a.OH != a.H || a.OW != a.W ||
      (a.fire_E[0] < 1 && a.fire_E[1] < 1) ||
      a.tiles_n < 1 || a.tiles_m != a.N * a.tiles_y * a.tiles_x || a.ntiles != a.tiles_m * a.tiles_n || a.grid < 1 ||
      a.in_sN < 0 || a.in_sH < 0 || a.in_sW < a.C)
    return (int)hipErrorInvalidValue;
  for (int e = 0; e < 2; ++e) {   // a part with no channels does not exist (a ConvX -> ConvY pair instead of a module)
    if (a.fire_E[e] == 0) continue;
    if (!a.fire_w[e] || !a.fire_scale[e] || !a.fire_shift[e] || !a.fire_out[e] || a.fire_E[e] < CE || a.fire_E[e] % CE != 0 ||
        a.fire_sP[e] < a.fire_E[e] || a.fire_sP[e] % CE != 0 || a.fire_sN[e] % CE != 0 || ((uintptr_t)a.fire_out[e] & 15) || ((uintptr_t)a.fire_w[e] & 15))
      return (int)hipErrorInvalidValue;
  }
  int ch, cw, pool_pos = 0;
  if (pool) {
    // max-pooling with windows of 2 or 3 at stride 2, no padding; every window starts inside the map
    if (a.pool != POOL_MAX || a.pk < 2 || a.pk > 3 || a.ps != 2 || a.pp != 0 || a.pph < 1 || a.ppw < 1 || a.PH < 1 || a.PW < 1 ||
        (a.PH - 1) * a.ps >= a.H || (a.PW - 1) * a.ps >= a.W ||
        a.tiles_y != (a.PH + a.pph - 1) / a.pph || a.tiles_x != (a.PW + a.ppw - 1) / a.ppw)
      return (int)hipErrorInvalidValue;
    ch = (a.pph - 1) * a.ps + a.pk; cw = (a.ppw - 1) * a.ps + a.pk;
    pool_pos = ch * cw;
  } else {
    if (a.th < 1 || a.tw < 1 || a.tiles_y != (a.H + a.th - 1) / a.th || a.tiles_x != (a.W + a.tw - 1) / a.tw) return (int)hipErrorInvalidValue;
    ch = a.th; cw = a.tw;
  }
  const int ring = a.fire_E[1] > 0 ? 1 : 0;
  const int positions = (ch + 2 * ring) * (cw + 2 * ring);
  const int lds = fire_lds(positions, a.K, ESZ, pool_pos);
  if (positions > kFireMaxPositions || lds > 160 * 1024) return (int)hipErrorInvalidValue;
  if (first3) return pool ? launch_fire_inst<T, true, 9>(a, lds, st) : launch_fire_inst<T, false, 9>(a, lds, st);
  return pool ? launch_fire_inst<T, true, 1>(a, lds, st) : launch_fire_inst<T, false, 1>(a, lds, st);
}

int launch_fire(const ConvArgs& a, int dtype, void* stream) {
  return dtype == DT_BF16 ? launch_fire_t<bf16_t>(a, (hipStream_t)stream) : launch_fire_t<float>(a, (hipStream_t)stream);
}

size_t fire_lds_bytes(int conv_h, int conv_w, int S, int esz, int pooled, int ring) {
  return (size_t)fire_lds((conv_h + 2 * ring) * (conv_w + 2 * ring), S, esz, pooled ? conv_h * conv_w : 0);
}

}  // namespace xenos
