// int4-weight x int8-activation linear layer of the quantised attention block (Section 4.2: per-channel
// symmetric weights, per-token symmetric activations):
//   out[m,n] = (sum_k x[m,k] * w[n,k]) * s_x[m] * s_w[n],   M <= 64 tokens (a decode batch).
//
// At decode batch sizes the layer is bound by reading the weights once, so the work is cut into many small
// workgroups: one per 16 output channels, whose 8 wavefronts split the contraction and add up through LDS.
// V_MFMA_I32_16X16X64_I8 takes the activations as the A operand (row = token) and the weights as the B operand
// (column = output channel); D: lane L, register v -> token 4*(L/16) + v, channel L%16.
// Only the pairing of A and B bytes matters for a dot product, not their order, so the nibbles are never
// interleaved back: a lane's 16 weight bytes give one operand of the even k (low nibbles) and one of the odd k
// (high nibbles), and the activation bytes are split the same way with byte permutes.
// A nibble is moved to the TOP of its byte, which sign-extends it for free and scales it by 16; the int32 sum is
// therefore 16 x the true one (still exact: |16 w| <= 128, |x| <= 127, K up to 2^16) and is shifted back at the end.
#include "wsvd_dev.h"
#include "wsvd_internal.h"

namespace {

constexpr int kLinWaves = 8;
constexpr int kLinStepK = 256;     // contraction elements per wave step: 4 lane groups x 64
constexpr int kLinU = 2;           // steps in flight per wave

WSVD_DEV v4i mfma16(v4i a, v4i b, v4i c) { return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0); }

// even / odd bytes of 8 consecutive dwords (32 bytes) -> two operands of 16 bytes
WSVD_DEV void split_even_odd(const v4i lo, const v4i hi, v4i& even, v4i& odd) {
  even[0] = __builtin_amdgcn_perm(lo[1], lo[0], 0x06040200u); odd[0] = __builtin_amdgcn_perm(lo[1], lo[0], 0x07050301u);
  even[1] = __builtin_amdgcn_perm(lo[3], lo[2], 0x06040200u); odd[1] = __builtin_amdgcn_perm(lo[3], lo[2], 0x07050301u);
  even[2] = __builtin_amdgcn_perm(hi[1], hi[0], 0x06040200u); odd[2] = __builtin_amdgcn_perm(hi[1], hi[0], 0x07050301u);
  even[3] = __builtin_amdgcn_perm(hi[3], hi[2], 0x06040200u); odd[3] = __builtin_amdgcn_perm(hi[3], hi[2], 0x07050301u);
}

// The two halves every variant of the layer shares.  Output coordinates of a thread in the final pass and their
// scales are requested at the very start and used at the very end; the final pass adds the waves' partial sums
// (slot k of wave w at red[w * wave_stride + k], k = ((tile * MB + block) * 64 + lane) * 4 + register), undoes the
// factor 16 and applies the two scales.  Thread -> (tile, token, channel), channel fastest, so a 16-lane group writes
// 64 contiguous bytes.
template <int MB, int NC>
struct LinScales {
  static constexpr int NOUT = NC * MB * 256;
  static constexpr int OPT = (NOUT + kLinWaves * 64 - 1) / (kLinWaves * 64);
  float sx[OPT], sw[OPT];
};

template <int MB, int NC>
WSVD_DEV void linear_scales(LinScales<MB, NC>& sc, const uint16_t* xs, const uint16_t* wsc, int n0, int M, int N) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int it = 0; it < LinScales<MB, NC>::OPT; it++) {
    const int o = min(it * kLinWaves * 64 + tid, LinScales<MB, NC>::NOUT - 1);
    const int c = o / (MB * 256), rem = o % (MB * 256);
    const int m = min((rem >> 8) * 16 + ((rem & 255) >> 4), M - 1);
    sc.sx[it] = f16_bits_to_f32(xs[m]);
    sc.sw[it] = f16_bits_to_f32(wsc[min(n0 + 16 * c + (o & 15), N - 1)]);
  }
}

template <int MB, int NC>
WSVD_DEV void linear_finish(const LinScales<MB, NC>& sc, const int* red, int wave_stride, int n0, int M, int N, float* out,
                            int N1, float* out2) {
  const int tid = threadIdx.x;
#pragma unroll
  for (int it = 0; it < LinScales<MB, NC>::OPT; it++) {
    const int o = it * kLinWaves * 64 + tid;
    if (o >= LinScales<MB, NC>::NOUT) break;
    const int c = o / (MB * 256), rem0 = o % (MB * 256);
    const int mb = rem0 >> 8, rem = rem0 & 255;
    const int ch = rem & 15, rr = rem >> 4;
    const int src_lane = (rr >> 2) * 16 + ch, v = rr & 3;
    int sum = 0;
#pragma unroll
    for (int k = 0; k < kLinWaves; k++) sum += red[k * wave_stride + ((c * MB + mb) * 64 + src_lane) * 4 + v];
    const int m = mb * 16 + rr;
    const int nt = n0 + 16 * c;
    // output columns [0, N1) form one row-major matrix, [N1, N) a second one (a 16-column tile never straddles)
    float* dst = nt < N1 ? out + (size_t)m * N1 + nt : out2 + (size_t)m * (N - N1) + (nt - N1);
    if (m < M && nt < N) dst[ch] = (float)(sum >> 4) * sc.sx[it] * sc.sw[it];
  }
}

// MB = blocks of 16 tokens (M <= 16 * MB); NC = tiles of 16 output channels per workgroup (2 when there are plenty of
// channels: the activations, which every workgroup reads in full from L2, are then fetched half as often).
// k order inside a 256-element wave step: lane group g takes [32 g, 32 g + 32) and [128 + 32 g, 128 + 32 g + 32), so
// that one load instruction covers 64 contiguous bytes of each of its 16 weight rows, and the four 16-byte pieces an
// activation load takes from a row fall into one 128-byte line.
template <int MB, int NC>
__global__ __launch_bounds__(kLinWaves * 64) void k_linear_w4a8(const int8_t* __restrict__ x, const uint16_t* __restrict__ xs,
                                                               const uint8_t* __restrict__ w, const uint16_t* __restrict__ wsc,
                                                               int M, int K, int N, float* __restrict__ out,
                                                               int N1, float* __restrict__ out2) {
  __shared__ int red[kLinWaves][NC][MB][64][4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n0 = blockIdx.x * 16 * NC;
  const int col = lane & 15, grp = lane >> 4;
  const int n_steps = (K + kLinStepK - 1) / kLinStepK;
  const uint8_t* wrow[NC];
#pragma unroll
  for (int c = 0; c < NC; c++) wrow[c] = w + (size_t)min(n0 + 16 * c + col, N - 1) * (size_t)(K >> 1);
  const int8_t* xrow[MB];
#pragma unroll
  for (int mb = 0; mb < MB; mb++) xrow[mb] = x + (size_t)min(mb * 16 + col, M - 1) * (size_t)K;

  LinScales<MB, NC> sc;
  linear_scales<MB, NC>(sc, xs, wsc, n0, M, N);

  v4i acc[NC][MB];
#pragma unroll
  for (int c = 0; c < NC; c++)
#pragma unroll
    for (int mb = 0; mb < MB; mb++) acc[c][mb] = v4i{0, 0, 0, 0};

  for (int s0 = wave; s0 < n_steps; s0 += kLinWaves * kLinU) {
    v4i wr[kLinU][NC][2], xr[kLinU][MB][4];
    // all loads of the batch first (addresses clamped into the row; a half group past K is masked below)
#pragma unroll
    for (int u = 0; u < kLinU; u++) {
      const int kb = (s0 + u * kLinWaves) * kLinStepK + 32 * grp;
      const int kc0 = min(kb, K - 32), kc1 = min(kb + 128, K - 32);
      // the two halves of a row's 128-byte line back to back (they merge into one fetch), activations afterwards
#pragma unroll
      for (int c = 0; c < NC; c++) {
        wr[u][c][0] = __builtin_nontemporal_load((const v4i*)(wrow[c] + (kc0 >> 1)));
        wr[u][c][1] = __builtin_nontemporal_load((const v4i*)(wrow[c] + (kc1 >> 1)));
      }
#pragma unroll
      for (int mb = 0; mb < MB; mb++) {
        xr[u][mb][0] = *(const v4i*)(xrow[mb] + kc0);
        xr[u][mb][1] = *(const v4i*)(xrow[mb] + kc0 + 16);
        xr[u][mb][2] = *(const v4i*)(xrow[mb] + kc1);
        xr[u][mb][3] = *(const v4i*)(xrow[mb] + kc1 + 16);
      }
    }
    // keep the whole batch in flight: without this the scheduler sinks most loads below the first products to save
    // registers, which turns one memory round trip into four
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < kLinU; u++) {
      const int kb = (s0 + u * kLinWaves) * kLinStepK + 32 * grp;
#pragma unroll
      for (int h = 0; h < 2; h++) {
        const uint32_t top = (kb + 128 * h < K) ? 0xF0F0F0F0u : 0u;
        v4i xe[MB], xo[MB];
#pragma unroll
        for (int mb = 0; mb < MB; mb++) split_even_odd(xr[u][mb][2 * h], xr[u][mb][2 * h + 1], xe[mb], xo[mb]);
#pragma unroll
        for (int c = 0; c < NC; c++) {
          v4i wlo, whi;
#pragma unroll
          for (int i = 0; i < 4; i++) {
            const uint32_t raw = (uint32_t)wr[u][c][h][i];
            wlo[i] = (int)((raw << 4) & top);   // 16 * w[even k]
            whi[i] = (int)(raw & top);          // 16 * w[odd k]
          }
#pragma unroll
          for (int mb = 0; mb < MB; mb++) {
            acc[c][mb] = mfma16(xe[mb], wlo, acc[c][mb]);
            acc[c][mb] = mfma16(xo[mb], whi, acc[c][mb]);
          }
        }
      }
    }
  }
#pragma unroll
  for (int c = 0; c < NC; c++)
#pragma unroll
    for (int mb = 0; mb < MB; mb++)
#pragma unroll
      for (int v = 0; v < 4; v++) red[wave][c][mb][lane][v] = acc[c][mb][v];
  __syncthreads();
  linear_finish<MB, NC>(sc, &red[0][0][0][0][0], NC * MB * 256, n0, M, N, out, N1, out2);
}

// The same layer with both operands staged through wave-private LDS.  The matrix-core layout wants lane = (row, k
// group), which read straight from row-major memory makes every load instruction touch 16 rows in 16- or 64-byte
// pieces.  Here a wave fetches its step of the weights (16 rows x 128 bytes per tile) and of the activations (16 rows x
// 256 bytes per token block) with whole 128-byte lines per row, writes them to its own LDS region and reads them back
// in operand order.  Row strides of 144 and 272 bytes spread both access patterns evenly over the banks.  No
// workgroup barrier is involved: a wave only ever touches its own region until the final reduction, whose per-wave
// slots live inside that region too.  For M <= 32.
constexpr int kLinWRow = 144, kLinXRow = 272;
template <int MB, int NC>
__global__ __launch_bounds__(kLinWaves * 64) void k_linear_w4a8_staged(const int8_t* __restrict__ x, const uint16_t* __restrict__ xs,
                                                                      const uint8_t* __restrict__ w, const uint16_t* __restrict__ wsc,
                                                                      int M, int K, int N, float* __restrict__ out,
                                                                      int N1, float* __restrict__ out2) {
  constexpr int WBYTES = 16 * kLinWRow, XBYTES = 16 * kLinXRow;
  constexpr int WAVE_LDS = NC * WBYTES + MB * XBYTES;
  static_assert(WAVE_LDS >= NC * MB * 1024 && WAVE_LDS % 16 == 0, "the reduction slots must fit into a wave's region");
  __shared__ __attribute__((aligned(16))) uint8_t lds[kLinWaves][WAVE_LDS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n0 = blockIdx.x * 16 * NC;
  const int col = lane & 15, grp = lane >> 4;
  const int n_steps = (K + kLinStepK - 1) / kLinStepK;
  uint8_t* my = lds[wave];
  // fetch coordinates: weights 8 rows x 8 pieces of 16 bytes per instruction, activations 4 rows x 16 pieces
  const int wr_row = lane >> 3, wr_piece = lane & 7;
  const int xr_row = lane >> 4, xr_piece = lane & 15;
  const uint8_t* wsrc[NC][2];
#pragma unroll
  for (int c = 0; c < NC; c++)
#pragma unroll
    for (int i = 0; i < 2; i++) wsrc[c][i] = w + (size_t)min(n0 + 16 * c + 8 * i + wr_row, N - 1) * (size_t)(K >> 1);
  const int8_t* xsrc[MB][4];
#pragma unroll
  for (int mb = 0; mb < MB; mb++)
#pragma unroll
    for (int i = 0; i < 4; i++) xsrc[mb][i] = x + (size_t)min(mb * 16 + 4 * i + xr_row, M - 1) * (size_t)K;

  LinScales<MB, NC> sc;
  linear_scales<MB, NC>(sc, xs, wsc, n0, M, N);

  v4i acc[NC][MB];
#pragma unroll
  for (int c = 0; c < NC; c++)
#pragma unroll
    for (int mb = 0; mb < MB; mb++) acc[c][mb] = v4i{0, 0, 0, 0};

  for (int s0 = wave; s0 < n_steps; s0 += kLinWaves * kLinU) {
    v4i wg[kLinU][NC][2], xg[kLinU][MB][4];
    // all fetches of the batch first; a piece past the end of the row is fetched from the row's last 16 bytes instead
    // (its products are masked below)
#pragma unroll
    for (int u = 0; u < kLinU; u++) {
      const int step = s0 + u * kLinWaves;
      const int wo = min(step * (kLinStepK / 2) + wr_piece * 16, (K >> 1) - 16);
      const int xo = min(step * kLinStepK + xr_piece * 16, K - 16);
#pragma unroll
      for (int c = 0; c < NC; c++)
#pragma unroll
        for (int i = 0; i < 2; i++) wg[u][c][i] = __builtin_nontemporal_load((const v4i*)(wsrc[c][i] + wo));
#pragma unroll
      for (int mb = 0; mb < MB; mb++)
#pragma unroll
        for (int i = 0; i < 4; i++) xg[u][mb][i] = *(const v4i*)(xsrc[mb][i] + xo);
    }
    __builtin_amdgcn_sched_barrier(0);      // keep the whole batch in flight
#pragma unroll
    for (int u = 0; u < kLinU; u++) {
      const int kb = (s0 + u * kLinWaves) * kLinStepK + 32 * grp;
      // earlier reads of the region are done (same-wave LDS operations execute in order); fences for the compiler
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int c = 0; c < NC; c++)
#pragma unroll
        for (int i = 0; i < 2; i++) *(v4i*)(my + c * WBYTES + (8 * i + wr_row) * kLinWRow + wr_piece * 16) = wg[u][c][i];
#pragma unroll
      for (int mb = 0; mb < MB; mb++)
#pragma unroll
        for (int i = 0; i < 4; i++) *(v4i*)(my + NC * WBYTES + mb * XBYTES + (4 * i + xr_row) * kLinXRow + xr_piece * 16) = xg[u][mb][i];
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int h = 0; h < 2; h++) {
        const uint32_t top = (kb + 128 * h < K) ? 0xF0F0F0F0u : 0u;
        v4i xe[MB], xo2[MB];
#pragma unroll
        for (int mb = 0; mb < MB; mb++) {
          const uint8_t* xp = my + NC * WBYTES + mb * XBYTES + col * kLinXRow + 128 * h + 32 * grp;
          split_even_odd(*(const v4i*)xp, *(const v4i*)(xp + 16), xe[mb], xo2[mb]);
        }
#pragma unroll
        for (int c = 0; c < NC; c++) {
          const v4i raw4 = *(const v4i*)(my + c * WBYTES + col * kLinWRow + 64 * h + 16 * grp);
          v4i wlo, whi;
#pragma unroll
          for (int i = 0; i < 4; i++) {
            const uint32_t raw = (uint32_t)raw4[i];
            wlo[i] = (int)((raw << 4) & top);   // 16 * w[even k]
            whi[i] = (int)(raw & top);          // 16 * w[odd k]
          }
#pragma unroll
          for (int mb = 0; mb < MB; mb++) {
            acc[c][mb] = mfma16(xe[mb], wlo, acc[c][mb]);
            acc[c][mb] = mfma16(xo2[mb], whi, acc[c][mb]);
          }
        }
      }
    }
  }
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  int* redw = (int*)my;                       // [NC][MB][64][4], inside this wave's own region
#pragma unroll
  for (int c = 0; c < NC; c++)
#pragma unroll
    for (int mb = 0; mb < MB; mb++) *(v4i*)&redw[((c * MB + mb) * 64 + lane) * 4] = acc[c][mb];
  __syncthreads();
  linear_finish<MB, NC>(sc, (const int*)&lds[0][0], WAVE_LDS / 4, n0, M, N, out, N1, out2);
}

}  // namespace


hipError_t wsvd_launch_linear_w4a8(const int8_t* x, const void* x_scale, const void* w_i4, const void* w_scale, int64_t M,
                                   int64_t K, int64_t N, float* out, int64_t n_first, float* out2, bool direct, hipStream_t s) {
  if (M < 1 || M > 64 || K < 64 || K % 64 != 0 || K > 65536 || N % 16 != 0) return hipErrorInvalidValue;
  if (n_first < 0 || n_first > N || n_first % 16 != 0 || (n_first < N && !out2)) return hipErrorInvalidValue;
  const int N1 = (int)n_first;
  const uint16_t* xs = (const uint16_t*)x_scale;
  const uint16_t* ws = (const uint16_t*)w_scale;
  const uint8_t* w = (const uint8_t*)w_i4;
  const int mbk = (int)((M + 15) / 16);
  dim3 block(kLinWaves * 64);
  // two 16-channel tiles per workgroup once that still leaves a few workgroups per CU
  const bool two = N / 32 >= 512;
  dim3 grid((unsigned)(two ? (N + 31) / 32 : N / 16));
  if (mbk <= 2 && !direct) {
    if (mbk == 1 && two) hipLaunchKernelGGL((k_linear_w4a8_staged<1, 2>), grid, block, 0, s, x, xs, w, ws, (int)M, (int)K, (int)N, out, N1, out2);
    else if (mbk == 1) hipLaunchKernelGGL((k_linear_w4a8_staged<1, 1>), grid, block, 0, s, x, xs, w, ws, (int)M, (int)K, (int)N, out, N1, out2);
    else if (two) hipLaunchKernelGGL((k_linear_w4a8_staged<2, 2>), grid, block, 0, s, x, xs, w, ws, (int)M, (int)K, (int)N, out, N1, out2);
    else hipLaunchKernelGGL((k_linear_w4a8_staged<2, 1>), grid, block, 0, s, x, xs, w, ws, (int)M, (int)K, (int)N, out, N1, out2);
    return hipGetLastError();
  }
  if (mbk <= 2 && two) {
    if (mbk == 1) hipLaunchKernelGGL((k_linear_w4a8<1, 2>), grid, block, 0, s, x, xs, w, ws, (int)M, (int)K, (int)N, out, N1, out2);
    else hipLaunchKernelGGL((k_linear_w4a8<2, 2>), grid, block, 0, s, x, xs, w, ws, (int)M, (int)K, (int)N, out, N1, out2);
    return hipGetLastError();
  }
  grid = dim3((unsigned)(N / 16));
  switch (mbk) {
    case 1: hipLaunchKernelGGL((k_linear_w4a8<1, 1>), grid, block, 0, s, x, xs, w, ws, (int)M, (int)K, (int)N, out, N1, out2); break;
    case 2: hipLaunchKernelGGL((k_linear_w4a8<2, 1>), grid, block, 0, s, x, xs, w, ws, (int)M, (int)K, (int)N, out, N1, out2); break;
    case 3: hipLaunchKernelGGL((k_linear_w4a8<3, 1>), grid, block, 0, s, x, xs, w, ws, (int)M, (int)K, (int)N, out, N1, out2); break;
    default: hipLaunchKernelGGL((k_linear_w4a8<4, 1>), grid, block, 0, s, x, xs, w, ws, (int)M, (int)K, (int)N, out, N1, out2); break;
  }
  return hipGetLastError();
}
