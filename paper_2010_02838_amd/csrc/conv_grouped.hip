// Grouped convolution (the 3x3 of the aggregated-transformation networks that Section 5 of the paper pairs with
// ResNets) on top of the dense matrix-core kernels.
//
// Output channels [g*C/G, (g+1)*C/G) read input channels of the same range only (Cin = Cout = C here).  The channels
// are cut into slices of at most 128 (whole groups); inside a slice the convolution is run as a dense one whose
// filter is zero outside the groups' diagonal blocks, so that a slice is one ordinary [pixels][slice] x
// [slice][taps * slice] problem for conv_fprop_mfma / conv_dgrad_mfma / conv_wgrad_mfma.  Those kernels want
// contiguous tensors, so the activations are copied into slice-major form ([slice][pixel][channel of the slice])
// and back; the kernels of this file are these copies, the expansion of the grouped filter into the dense
// per-slice filters, and the extraction of the grouped filter gradient from the dense per-slice ones.
// The dense form spends (slice width / channels per group) times the arithmetic of the grouped convolution; what
// it buys is the matrix cores at the tile shapes they are good at.
#include "common.h"
#include "kernels.h"

namespace cd {

int grouped_slice_width(int C) { return C <= 128 ? C : 128; }

bool grouped_conv_supported(int C, int groups) {
  if (groups < 1 || C % groups) return false;
  const int cg = C / groups, sw = grouped_slice_width(C);
  return C % 8 == 0 && C % sw == 0 && sw % cg == 0;
}

namespace {

// [M][C] <-> [C / SW][M][SW], 16 bytes at a time.  TO_SLICES: gather; else scatter (adding to what is there if acc).
template <bool TO_SLICES>
__global__ void __launch_bounds__(256) slice_copy_k(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int64_t M,
                                                    int C, int SW, int acc) {
  const int vpr = C / 8, vps = SW / 8;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= M * vpr) return;
  const int64_t m = idx / vpr;
  const int v = (int)(idx - m * vpr);
  const int s = v / vps, vl = v - s * vps;
  const int64_t row_major = m * C + (int64_t)v * 8, slice_major = ((int64_t)s * M + m) * SW + (int64_t)vl * 8;
  if (TO_SLICES) {
    *reinterpret_cast<uint4*>(dst + slice_major) = *reinterpret_cast<const uint4*>(src + row_major);
  } else {
    uint4 val = *reinterpret_cast<const uint4*>(src + slice_major);
    if (acc) {
      const uint4 old = *reinterpret_cast<const uint4*>(dst + row_major);
      const uint32_t a[4] = {val.x, val.y, val.z, val.w}, b[4] = {old.x, old.y, old.z, old.w};
      uint32_t r[4];
#pragma unroll
      for (int q = 0; q < 4; q++) {
        const float lo = __uint_as_float(a[q] << 16) + __uint_as_float(b[q] << 16);
        const float hi = __uint_as_float(a[q] & 0xffff0000u) + __uint_as_float(b[q] & 0xffff0000u);
        r[q] = (uint32_t)f32_to_bf16(lo) | ((uint32_t)f32_to_bf16(hi) << 16);
      }
      val = make_uint4(r[0], r[1], r[2], r[3]);
    }
    *reinterpret_cast<uint4*>(dst + row_major) = val;
  }
}

// w [C][taps][cg] (grouped) -> wd [C / SW][SW][taps][SW] (dense per slice, zero outside the diagonal blocks)
__global__ void __launch_bounds__(256) expand_group_weights_k(const bf16_t* __restrict__ w, bf16_t* __restrict__ wd, int C,
                                                              int taps, int cg, int SW) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t n = (int64_t)C * taps * SW;
  if (idx >= n) return;
  const int il = (int)(idx % SW);                    // input channel inside the slice
  const int t = (int)((idx / SW) % taps);
  const int o = (int)(idx / ((int64_t)SW * taps));   // global output channel = slice * SW + local
  const int ol = o % SW;
  const bool same_group = il / cg == ol / cg;
  wd[idx] = same_group ? w[((int64_t)o * taps + t) * cg + il % cg] : (bf16_t)0;
}

// dwd [C / SW][SW][taps][SW] (dense per slice, fp32) -> dw [C][taps][cg]: the diagonal blocks
__global__ void __launch_bounds__(256) extract_group_dw_k(const float* __restrict__ dwd, float* __restrict__ dw, int C,
                                                          int taps, int cg, int SW) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t n = (int64_t)C * taps * cg;
  if (idx >= n) return;
  const int j = (int)(idx % cg);
  const int t = (int)((idx / cg) % taps);
  const int o = (int)(idx / ((int64_t)cg * taps));
  const int ol = o % SW;
  dw[idx] = dwd[((int64_t)o * taps + t) * SW + (ol / cg) * cg + j];
}

}  // namespace

void slices_gather(const bf16_t* x, bf16_t* xs, int64_t M, int C, hipStream_t s) {
  const int64_t n = M * (C / 8);
  hipLaunchKernelGGL(slice_copy_k<true>, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s, x, xs, M, C, grouped_slice_width(C), 0);
}

void slices_scatter(const bf16_t* xs, bf16_t* x, int64_t M, int C, bool accumulate, hipStream_t s) {
  const int64_t n = M * (C / 8);
  hipLaunchKernelGGL(slice_copy_k<false>, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s, xs, x, M, C,
                     grouped_slice_width(C), accumulate ? 1 : 0);
}

void expand_group_weights(const bf16_t* w, bf16_t* wd, int C, int taps, int groups, hipStream_t s) {
  const int64_t n = (int64_t)C * taps * grouped_slice_width(C);
  hipLaunchKernelGGL(expand_group_weights_k, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s, w, wd, C, taps, C / groups,
                     grouped_slice_width(C));
}

void extract_group_dw(const float* dwd, float* dw, int C, int taps, int groups, hipStream_t s) {
  const int64_t n = (int64_t)C * taps * (C / groups);
  hipLaunchKernelGGL(extract_group_dw_k, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s, dwd, dw, C, taps, C / groups,
                     grouped_slice_width(C));
}

}  // namespace cd
