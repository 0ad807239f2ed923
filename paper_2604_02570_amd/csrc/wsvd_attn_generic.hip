// Decode attention over F32 / BF16 latent caches (row-major planes), plain vector ALU.
//
// A latent row is rank*esize bytes; LPR = row_bytes/16 adjacent lanes share a row, each holding a
// 16-byte slice, so a wavefront load covers 64/LPR consecutive rows = 1 KiB of contiguous cache.
// Each lane group runs its own online softmax (running max, sum, latent-space accumulator) over the
// rows it streams; the groups are merged once at the end, like sequence splits.
#include "wsvd_attn_common.h"
#include "wsvd_internal.h"

template <int ESZ>
WSVD_DEV void unpack16(const v4i& raw, float* f) {
  if (ESZ == 4) {
#pragma unroll
    for (int i = 0; i < 4; i++) f[i] = __int_as_float(raw[i]);
  } else {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      f[2 * i] = __uint_as_float((uint32_t)raw[i] << 16);
      f[2 * i + 1] = __uint_as_float((uint32_t)raw[i] & 0xFFFF0000u);
    }
  }
}

constexpr int kMaxG = 8;

template <int ESZ, int R, int G>
__global__ __launch_bounds__(256) void k_attn_generic(AttnParams p) {
  constexpr int ROWB = R * ESZ;          // bytes per latent row
  constexpr int LPR = ROWB / 16;         // lanes per row
  constexpr int VPL = 16 / ESZ;          // values per lane
  constexpr int RPW = 64 / LPR;          // rows per wavefront load
  constexpr int NGRP = 4 * RPW;          // lane groups per workgroup
  constexpr int UNROLL = 4;

  constexpr int FIT = R * ESZ / 32;     // 16-byte staging passes for an R x 128 factor
  __shared__ v4i fac_lds[R * 128 * ESZ / 16];
  __shared__ __attribute__((aligned(16))) float q_lds[G * 128];
  __shared__ float qts[G * R];
  __shared__ float Msh[G], Lsh[G], Ush[G * R];
  __shared__ float gm[NGRP * G], gl[NGRP * G];
  __shared__ float gu[NGRP * G * R];
  // parts the merge of the NGRP lane groups is divided into (a power of two that divides NGRP; 1 = a single pass)
  constexpr int NPART = G * R >= 256 ? 1 : (256 / (G * R) >= 8 ? 8 : 256 / (G * R) >= 4 ? 4 : 2);
  static_assert(NGRP % NPART == 0, "the lane groups divide evenly over the parts");
  __shared__ float pm[NPART * G], pl[NPART * G], pu[NPART * G * R];
  __shared__ int flag_sh;

  const WorkItem w = decode_work(p, p.seq_lens[blockIdx.z]);
  if (w.n == 0) { write_zero_outputs(p, w); return; }
  if (!w.active) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int sl = lane % LPR;                       // which 16-byte slice of the row
  const int grp = wave * RPW + lane / LPR;         // lane group id within the workgroup

  const int fac16 = R * p.d * ESZ / 16;
  {
    StageRegs<FIT> st;
    QRegsT<(G * 128 + 255) / 256> qr;               // 256 query elements per pass
    stage_issue<FIT>(st, (const char*)p.BK + (size_t)w.kv * R * p.d * ESZ, fac16);
    q_issue(p, w.b, w.kv, qr);
    stage_commit<FIT>(st, fac_lds, fac16);
    q_commit(p, qr, q_scale_value(p, w.b, q_scale_raw(p, w.b)), q_lds);
  }
  __syncthreads();
  compute_qtilde<R, ESZ>(p, fac_lds, q_lds, qts);
  float qt[G][VPL];
#pragma unroll
  for (int g = 0; g < G; g++)
#pragma unroll
    for (int v = 0; v < VPL; v++) qt[g][v] = qts[g * R + sl * VPL + v];

  const size_t plane = ((size_t)w.b * p.Hkv + w.kv) * (size_t)p.t_cap * ROWB;
  const uint8_t* kb = p.k_codes + plane + sl * 16;
  const uint8_t* vb = p.v_codes + plane + sl * 16;

  float m[G], l[G], u[G][VPL];
#pragma unroll
  for (int g = 0; g < G; g++) {
    m[g] = -INFINITY; l[g] = 0.f;
#pragma unroll
    for (int v = 0; v < VPL; v++) u[g][v] = 0.f;
  }

  // Two batches of UNROLL rows per lane group in flight: the next batch is requested before the current one is
  // consumed, so a short chunk (640 rows = 3 batches) waits for memory twice, not three times: 8.3 -> 7.9 us for the
  // single 640-row bf16 sequence.  Rows are consumed in the same order as without the prefetch.  (Measured slower:
  // the first batches and B_V requested in front of the query absorption, 8.5-8.9 us.)
  constexpr int STEP = NGRP * UNROLL;
  auto load_rows = [&](v4i (&kr)[UNROLL], v4i (&vr)[UNROLL], int t0) {
#pragma unroll
    for (int k = 0; k < UNROLL; k++) {
      const int t = t0 + k * NGRP;
      if (t < w.row_end) {
        kr[k] = *(const v4i*)(kb + (size_t)t * ROWB);
        vr[k] = *(const v4i*)(vb + (size_t)t * ROWB);
      }
    }
  };
  auto use_rows = [&](const v4i (&kr)[UNROLL], const v4i (&vr)[UNROLL], int t0) {
#pragma unroll
    for (int k = 0; k < UNROLL; k++) {
      const int t = t0 + k * NGRP;
      if (t < w.row_end) {          // uniform within a lane group
        float kf[VPL], vf[VPL];
        unpack16<ESZ>(kr[k], kf);
        unpack16<ESZ>(vr[k], vf);
#pragma unroll
        for (int g = 0; g < G; g++) {
          float s = 0.f;
#pragma unroll
          for (int v = 0; v < VPL; v++) s = fmaf(qt[g][v], kf[v], s);
          s = group_sum<LPR>(s);
          const float mn = fmaxf(m[g], s);
          const float alpha = __builtin_amdgcn_exp2f(m[g] - mn);
          const float pw = __builtin_amdgcn_exp2f(s - mn);
          l[g] = fmaf(l[g], alpha, pw);
#pragma unroll
          for (int v = 0; v < VPL; v++) u[g][v] = fmaf(u[g][v], alpha, pw * vf[v]);
          m[g] = mn;
        }
      }
    }
  };
  {
    v4i ka[UNROLL], va[UNROLL], kb2[UNROLL], vb2[UNROLL];
    int t0 = w.row_begin + grp;
    load_rows(ka, va, t0);
    while (t0 < w.row_end) {
      load_rows(kb2, vb2, t0 + STEP);       // (nothing is requested past the chunk's end)
      use_rows(ka, va, t0);
      t0 += STEP;
      if (t0 >= w.row_end) break;
      load_rows(ka, va, t0 + STEP);
      use_rows(kb2, vb2, t0);
      t0 += STEP;
    }
  }
  // NOTE: group_sum uses DPP across the LPR lanes of a row; lanes of a group take the same branch
  // (t depends only on the group), so the exchanged values are always defined.

#pragma unroll
  for (int g = 0; g < G; g++) {
    if (sl == 0) { gm[grp * G + g] = m[g]; gl[grp * G + g] = l[g]; }
#pragma unroll
    for (int v = 0; v < VPL; v++) gu[(grp * G + g) * R + sl * VPL + v] = u[g][v];
  }
  __syncthreads();
  // Merge of the lane groups' partial results, one thread per (part of the groups, head, latent dim), then one per
  // (head, latent dim) over the parts: with a single head of rank 32 a lone pass would leave 224 of the 256 threads idle
  // while 32 walk 64 groups each.
  if constexpr (NPART > 1) {
    for (int i = tid; i < NPART * G * R; i += 256) {
      const int part = i / (G * R), g = (i / R) % G, j = i % R;
      const int k0 = part * (NGRP / NPART), k1 = k0 + NGRP / NPART;
      float M = -INFINITY;
      for (int k = k0; k < k1; k++) M = fmaxf(M, gm[k * G + g]);
      float L = 0.f, U = 0.f;
      for (int k = k0; k < k1; k++) {
        const float e = M == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(gm[k * G + g] - M);   // a part without any row
        L = fmaf(gl[k * G + g], e, L);
        U = fmaf(gu[(k * G + g) * R + j], e, U);
      }
      pu[i] = U;
      if (j == 0) { pm[part * G + g] = M; pl[part * G + g] = L; }
    }
    __syncthreads();
  }
  for (int i = tid; i < G * R; i += 256) {
    const int g = i / R, j = i % R;
    const float* sm = NPART > 1 ? pm : gm;
    const float* sl_ = NPART > 1 ? pl : gl;
    const float* su = NPART > 1 ? pu : gu;
    constexpr int NS = NPART > 1 ? NPART : NGRP;
    float M = -INFINITY;
    for (int k = 0; k < NS; k++) M = fmaxf(M, sm[k * G + g]);
    float L = 0.f, U = 0.f;
    for (int k = 0; k < NS; k++) {
      const float e = __builtin_amdgcn_exp2f(sm[k * G + g] - M);      // the workgroup holds at least one row: M is finite
      L = fmaf(sl_[k * G + g], e, L);
      U = fmaf(su[(k * G + g) * R + j], e, U);
    }
    Ush[i] = U;
    if (j == 0) { Msh[g] = M; Lsh[g] = L; }
  }
  {
    StageRegs<FIT> st;   // B_K is no longer needed: reuse its LDS for B_V
    stage_issue<FIT>(st, (const char*)p.BV + (size_t)w.kv * R * p.d * ESZ, fac16);
    stage_commit<FIT>(st, fac_lds, fac16);
  }
  __syncthreads();
  attn_tail<R, ESZ>(p, w, Msh, Lsh, Ush, &flag_sh, fac_lds);
}

template <int ESZ, int R>
static hipError_t launch_g(const AttnParams& p, dim3 grid, hipStream_t s) {
  switch (p.G) {
    case 1: hipLaunchKernelGGL((k_attn_generic<ESZ, R, 1>), grid, dim3(256), 0, s, p); break;
    case 2: hipLaunchKernelGGL((k_attn_generic<ESZ, R, 2>), grid, dim3(256), 0, s, p); break;
    case 3: hipLaunchKernelGGL((k_attn_generic<ESZ, R, 3>), grid, dim3(256), 0, s, p); break;
    case 4: hipLaunchKernelGGL((k_attn_generic<ESZ, R, 4>), grid, dim3(256), 0, s, p); break;
    case 5: hipLaunchKernelGGL((k_attn_generic<ESZ, R, 5>), grid, dim3(256), 0, s, p); break;
    case 6: hipLaunchKernelGGL((k_attn_generic<ESZ, R, 6>), grid, dim3(256), 0, s, p); break;
    case 7: hipLaunchKernelGGL((k_attn_generic<ESZ, R, 7>), grid, dim3(256), 0, s, p); break;
    case 8: hipLaunchKernelGGL((k_attn_generic<ESZ, R, 8>), grid, dim3(256), 0, s, p); break;
    default: return hipErrorNotSupported;
  }
  return hipGetLastError();
}

hipError_t wsvd_launch_attn_generic(const AttnParams& p, int latent_dtype, int rank, dim3 grid, hipStream_t s) {
  if (latent_dtype == WSVD_F32) {
    if (rank == 16) return launch_g<4, 16>(p, grid, s);
    if (rank == 32) return launch_g<4, 32>(p, grid, s);
    if (rank == 64) return launch_g<4, 64>(p, grid, s);
  } else if (latent_dtype == WSVD_BF16) {
    if (rank == 16) return launch_g<2, 16>(p, grid, s);
    if (rank == 32) return launch_g<2, 32>(p, grid, s);
    if (rank == 64) return launch_g<2, 64>(p, grid, s);
  }
  return hipErrorInvalidValue;
}
