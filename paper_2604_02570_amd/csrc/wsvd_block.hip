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

// MB = blocks of 16 tokens (M <= 16 * MB)
template <int MB>
__global__ __launch_bounds__(kLinWaves * 64) void k_linear_w4a8(const int8_t* __restrict__ x, const uint16_t* __restrict__ xs,
                                                               const uint8_t* __restrict__ w, const uint16_t* __restrict__ wsc,
                                                               int M, int K, int N, float* __restrict__ out,
                                                               int N1, float* __restrict__ out2) {
  __shared__ int red[kLinWaves][MB][64][4];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n0 = blockIdx.x * 16;
  const int col = lane & 15, grp = lane >> 4;
  const int n_steps = (K + kLinStepK - 1) / kLinStepK;
  const uint8_t* wrow = w + (size_t)(n0 + col) * (size_t)(K >> 1);
  const int8_t* xrow[MB];
#pragma unroll
  for (int mb = 0; mb < MB; mb++) xrow[mb] = x + (size_t)min(mb * 16 + col, M - 1) * (size_t)K;

  // output coordinates of this thread in the final pass, and their scales (requested now, used at the very end)
  constexpr int OPT = (MB * 256 + kLinWaves * 64 - 1) / (kLinWaves * 64);
  float sx[OPT], sw[OPT];
#pragma unroll
  for (int it = 0; it < OPT; it++) {
    const int o = min(it * kLinWaves * 64 + tid, MB * 256 - 1);
    const int m = min((o >> 8) * 16 + ((o & 255) >> 4), M - 1);
    sx[it] = f16_bits_to_f32(xs[m]);
    sw[it] = f16_bits_to_f32(wsc[n0 + (o & 15)]);
  }

  v4i acc[MB];
#pragma unroll
  for (int mb = 0; mb < MB; mb++) acc[mb] = v4i{0, 0, 0, 0};

  for (int s0 = wave; s0 < n_steps; s0 += kLinWaves * kLinU) {
    v4i wr[kLinU][2], xr[kLinU][MB][4];
    // all loads of the batch first (addresses clamped into the row; a group past K is masked below)
#pragma unroll
    for (int u = 0; u < kLinU; u++) {
      const int k = (s0 + u * kLinWaves) * kLinStepK + 64 * grp;
      const int kc = min(k, K - 64);
      wr[u][0] = __builtin_nontemporal_load((const v4i*)(wrow + (kc >> 1)));
      wr[u][1] = __builtin_nontemporal_load((const v4i*)(wrow + (kc >> 1) + 16));
#pragma unroll
      for (int mb = 0; mb < MB; mb++)
#pragma unroll
        for (int i = 0; i < 4; i++) xr[u][mb][i] = *(const v4i*)(xrow[mb] + kc + 16 * i);
    }
    // keep the whole batch in flight: without this the scheduler sinks most loads below the first products to save
    // registers, which turns one memory round trip into four
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < kLinU; u++) {
      const int k = (s0 + u * kLinWaves) * kLinStepK + 64 * grp;
      const bool on = k < K;
      const uint32_t top = on ? 0xF0F0F0F0u : 0u;
      v4i wlo[2], whi[2];
#pragma unroll
      for (int h = 0; h < 2; h++)
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const uint32_t raw = (uint32_t)wr[u][h][i];
          wlo[h][i] = (int)((raw << 4) & top);   // 16 * w[even k]
          whi[h][i] = (int)(raw & top);          // 16 * w[odd k]
        }
#pragma unroll
      for (int mb = 0; mb < MB; mb++) {
        v4i xe, xo;
        split_even_odd(xr[u][mb][0], xr[u][mb][1], xe, xo);
        acc[mb] = mfma16(xe, wlo[0], acc[mb]);
        acc[mb] = mfma16(xo, whi[0], acc[mb]);
        split_even_odd(xr[u][mb][2], xr[u][mb][3], xe, xo);
        acc[mb] = mfma16(xe, wlo[1], acc[mb]);
        acc[mb] = mfma16(xo, whi[1], acc[mb]);
      }
    }
  }
#pragma unroll
  for (int mb = 0; mb < MB; mb++)
#pragma unroll
    for (int v = 0; v < 4; v++) red[wave][mb][lane][v] = acc[mb][v];
  __syncthreads();
  // thread -> (token, channel), channel fastest so a 16-lane group writes 64 contiguous bytes
#pragma unroll
  for (int it = 0; it < OPT; it++) {
    const int o = it * kLinWaves * 64 + tid;
    if (o >= MB * 256) break;
    const int mb = o >> 8, rem = o & 255;
    const int c = rem & 15, rr = rem >> 4;
    const int src_lane = (rr >> 2) * 16 + c, v = rr & 3;
    int sum = 0;
#pragma unroll
    for (int k = 0; k < kLinWaves; k++) sum += red[k][mb][src_lane][v];
    const int m = mb * 16 + rr;
    // output columns [0, N1) form one row-major matrix, [N1, N) a second one (a 16-column tile never straddles)
    float* dst = n0 < N1 ? out + (size_t)m * N1 + n0 : out2 + (size_t)m * (N - N1) + (n0 - N1);
    if (m < M) dst[c] = (float)(sum >> 4) * sx[it] * sw[it];
  }
}

}  // namespace

hipError_t wsvd_launch_linear_w4a8(const int8_t* x, const void* x_scale, const void* w_i4, const void* w_scale, int64_t M,
                                   int64_t K, int64_t N, float* out, int64_t n_first, float* out2, hipStream_t s) {
  if (M < 1 || M > 64 || K < 64 || K % 64 != 0 || K > 65536 || N % 16 != 0) return hipErrorInvalidValue;
  if (n_first < 0 || n_first > N || n_first % 16 != 0 || (n_first < N && !out2)) return hipErrorInvalidValue;
  const int N1 = (int)n_first;
  dim3 grid((unsigned)(N / 16)), block(kLinWaves * 64);
  const uint16_t* xs = (const uint16_t*)x_scale;
  const uint16_t* ws = (const uint16_t*)w_scale;
  const uint8_t* w = (const uint8_t*)w_i4;
  switch ((M + 15) / 16) {
    case 1: hipLaunchKernelGGL((k_linear_w4a8<1>), grid, block, 0, s, x, xs, w, ws, (int)M, (int)K, (int)N, out, N1, out2); break;
    case 2: hipLaunchKernelGGL((k_linear_w4a8<2>), grid, block, 0, s, x, xs, w, ws, (int)M, (int)K, (int)N, out, N1, out2); break;
    case 3: hipLaunchKernelGGL((k_linear_w4a8<3>), grid, block, 0, s, x, xs, w, ws, (int)M, (int)K, (int)N, out, N1, out2); break;
    default: hipLaunchKernelGGL((k_linear_w4a8<4>), grid, block, 0, s, x, xs, w, ws, (int)M, (int)K, (int)N, out, N1, out2); break;
  }
  return hipGetLastError();
}
