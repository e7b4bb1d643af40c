// bf16 implicit-GEMM convolution on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32
// accumulation.  These are the contractions of the forward and backward passes of the paper's
// networks (Section 3: ResNet50): fprop, dgrad and wgrad of every convolution.
//
//   fprop  y[m][n]  = sum_k im2col(x)[m][k] * w[n][k]          m = (b,ho,wo), k = (r,s,c)
//   dgrad  dx[m][c] = sum_k gather(dy)[m][k] * wt[c][k]        m = (b,h,w),   k = (r,s,n)
//   wgrad  dw[n][k] = sum_m dy[m][n] * im2col(x)[m][k]
//
// fprop and dgrad share one kernel: both operands are contiguous along the contraction index, so
// a lane's 8-element MFMA operand is one 16-byte load.  Block = 4 waves; buffer loads write global
// memory straight into LDS (three stages of unpadded, XOR-swizzled 64-byte rows: conflict-free
// 16-byte reads) -> MFMA; the fp32 tile is rounded to bf16, transposed through LDS and written as
// full 16-byte vectors along the channels.  The MFMA "A" operand is the filter tile and "B" the
// activation tile, so that a lane's 16 accumulators run along the output channels of one pixel.
#include "kernels.h"
#include <algorithm>

namespace cd {

#define CD_LDS __attribute__((address_space(3)))
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int BK = 32;  // contraction elements per main-loop step (one 64-byte LDS row)

struct IgemmArgs {
  const bf16_t* src;  // gathered tensor [B][Hs][Ws][Cs]
  const bf16_t* wt;   // [N][K], K = kh*kw*Cs, laid out (r, s, c)
  bf16_t* dst;        // [M][N]
  int64_t M;
  int N, K;
  int Hs, Ws, Cs, Hd, Wd, kh, kw, stride, pad, pad_w;
  // output row m = (b, hd, wd) is written to row (b*Ho + hd*omul + ooff_h)*Wo + wd*omul + ooff_w of dst
  int omul, ooff_h, ooff_w, Ho, Wo;
  int accumulate;     // the result is added to what dst holds, or to `addend` when that is set
  // accumulate only (nullable): a second tensor [M][N] added instead of the old contents of dst, and
  // (nullable) its gate, one bit per element (bit k of byte i gates element 8i + k): a cleared bit
  // drops the addend's element.  Lets a data gradient pick up the gated gradient of a residual branch
  // without that branch's gradient ever being written out.
  const bf16_t* addend = nullptr;
  const uint8_t* addend_gate = nullptr;
  // (nullable) a tensor [M][N] of which the output is the gradient behind a ReLU: output elements whose element
  // of relu_out is not positive are written as zero (the ReLU's backward pass, without a pass of its own)
  const bf16_t* relu_out = nullptr;
  // Grouped convolutions (sliced launches): the gathered tensor has src_pitch channels per pixel, of which column tile
  // tn reads the Cs = BN channels [tn * BN, (tn + 1) * BN): the slice of channels whose groups the tile's output
  // channels belong to.  The filter rows then hold kh * kw * Cs elements, zero outside a row's own group.
  int src_pitch = 0;   // 0: Cs (an ordinary convolution)
  int sliced = 0;
  int pointwise;  // kh = kw = 1, stride 1, no padding (set by the launcher)
  int group_m;    // GROUP kernels: tile order in groups of this many row tiles
  int ntiles;
  uint32_t src_bytes, wt_bytes;
  const bf16_t* bias;  // per-column bias added to the output (kernels with EPI >= 1)
  float* stat_partials;  // STATS kernels: [m-tiles][stat_pitch(N)] per-tile column sums and sums of squares
  // STATS == 2 (a data gradient that completes the gradient of a BatchNorm's output): the sums that BatchNorm's
  // backward pass reduces over the rows, taken from the values as they are stored: dz = the output, gated by the
  // BatchNorm's ReLU bit mask (bn_mask, nullable: no ReLU), and dz * xhat with xhat = (bn_x - mean) * invstd,
  // bn_x [M][N] the BatchNorm's input, bn_stats = [mean[N] | invstd[N]].  Written to stat_partials like the forward sums.
  const bf16_t* bn_x = nullptr;
  const uint8_t* bn_mask = nullptr;
  const float* bn_stats = nullptr;
};

int g_tune_tile = 0, g_tune_co = -1;  // tuning knobs of the microbenchmark

// Blocks are handed to the 8 XCDs round-robin; renumber so that consecutive logical tiles (which
// share activation rows and halos) run on the same XCD and meet in its L2.
__device__ inline unsigned xcd_remap(unsigned bid, unsigned nblocks) {
  const unsigned xcd = bid & 7u, idx = bid >> 3;
  const unsigned per = nblocks >> 3, rem = nblocks & 7u;
  return xcd * per + (xcd < rem ? xcd : rem) + idx;
}

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
// two floats -> two bf16 (round to nearest even) in one instruction
__device__ inline uint32_t pack_bf16x2(float a, float b) {
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));

// Element (c, c) of a 32x32 accumulator tile held in the MFMA output layout (the lane owns column
// lane % 32; register v holds row 8 (v / 4) + 4 (lane / 32) + v % 4), for c = lane % 32: register
// 4 (c / 8) + c % 4, picked by a select tree.  Only the half-wave with lane / 32 == (c / 4) % 2 holds it.
__device__ inline float tile_diagonal(f32x16_t d, int c) {
  const bool b0 = (c & 1) != 0, b1 = (c & 2) != 0, b3 = (c & 8) != 0, b4 = (c & 16) != 0;
  const float u0 = b0 ? d[1] : d[0], u1 = b0 ? d[3] : d[2], u2 = b0 ? d[5] : d[4], u3 = b0 ? d[7] : d[6];
  const float u4 = b0 ? d[9] : d[8], u5 = b0 ? d[11] : d[10], u6 = b0 ? d[13] : d[12], u7 = b0 ? d[15] : d[14];
  const float w0 = b1 ? u1 : u0, w1 = b1 ? u3 : u2, w2 = b1 ? u5 : u4, w3 = b1 ? u7 : u6;
  const float x0 = b3 ? w1 : w0, x1 = b3 ? w3 : w2;
  return b4 ? x1 : x0;
}

// 16-byte load through a raw buffer descriptor: an offset at or beyond the buffer size returns
// zeros, so a masked-out vector costs one select instead of a branch around the load.
typedef int v4i32_t __attribute__((ext_vector_type(4)));
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
__device__ inline uint4 buf_load16(__amdgpu_buffer_rsrc_t r, uint32_t byte_off) {
  const v4i32_t v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0);
  return make_uint4((uint32_t)v.x, (uint32_t)v.y, (uint32_t)v.z, (uint32_t)v.w);
}

// 16 bytes per lane from a buffer straight into LDS: lane l of the wave writes its vector at
// lds_addr + 16*l (lds_addr is uniform over the wave and travels in M0); an offset outside the
// buffer writes zeros.  The compiler does not see these loads: the kernel waits for them itself
// (wait_vmem) before a barrier publishes the tile.
typedef int rsrc_words_t __attribute__((ext_vector_type(4)));
// the four descriptor words of a raw buffer (stride 0): base address, size in bytes, data format
__device__ inline rsrc_words_t make_rsrc_words(const void* p, uint32_t bytes) {
  const uint64_t b = reinterpret_cast<uint64_t>(p);
  rsrc_words_t w;
  w.x = (int)(uint32_t)b;
  w.y = (int)((uint32_t)(b >> 32) & 0xffffu);
  w.z = (int)bytes;
  w.w = 0x00020000;
  return w;
}
__device__ inline void load_lds16(rsrc_words_t w, uint32_t lds_addr, uint32_t byte_off) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
               :
               : "s"(lds_addr), "v"(byte_off), "s"(w)
               : "memory");  // M0 cannot be named as a clobber: the compiler treats it as a reserved register (it rejects
                             // "m0" in a clobber list as such), i.e. it never keeps a value in M0 from one statement to
                             // the next and writes M0 itself right before each of its own uses
}
// wait until at most N of this wave's vector memory loads are outstanding
template <int N>
__device__ inline void wait_vmem() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// LDS tiles are [row][32 elements] = 64-byte rows without padding; the 16-byte column cv of a row
// is stored at column cv ^ ((row >> 2) & 3), which makes both the 16-byte stores (4 lanes per row)
// and the MFMA fragment reads (16 consecutive rows, one column) bank-conflict free.
__device__ inline int lds_off(int row, int cv) { return row * BK + ((cv ^ ((row >> 2) & 3)) << 3); }

// MODE 0: fprop gather, hs = hd*stride - pad + r.
// MODE 1: dgrad gather for stride 1, hs = hd + pad - r.
// (The dgrad of a stride-2 convolution is run as four MODE 0 problems, one per parity of the output
// pixel; see conv_dgrad_mfma.)
//
// Main loop: one barrier per 32-wide step.  At step kt the waves wait for their own loads of tile kt
// (issued two steps earlier), meet at the barrier, issue the loads of tile kt+2 into the stage that
// tile kt-1 occupied, read the fragments of tile kt and multiply.  The loads are inline assembly: the
// compiler does not track them, so it cannot serialise them against the LDS reads.
// F32OUT: the output is fp32 [M][N] (dense layers that produce logits); like the bf16 output it is
// transposed through LDS so that a store instruction writes whole 256-byte row segments.
// STATS 1: the epilogue also emits, per m-tile, the column sums and sums of squares of the bf16 values
// it writes (taken from the staged rows with transposing LDS reads and two MFMAs per fragment): the
// BatchNorm that follows a convolution gets its batch statistics without re-reading the tensor.
// STATS 2 (data gradients): per m-tile, the column sums of dz and dz * xhat that the backward pass of the BatchNorm
// whose output gradient this launch completes would otherwise reduce from memory (see IgemmArgs::bn_x).
// NWRAP: 1 when the gathered tensor has at least 32 channels (a 32-element step crosses at most one
// tap boundary), 4 for 8..31 channels.
// REMAP: output rows are placed with the strided row map of IgemmArgs (parity class of a stride-2 dgrad).
// EPI: 0 plain output, 1 per-column bias added, 2 bias and ReLU.  GROUP: grouped tile order (wide outputs).
// Both are compile-time: the plain kernels pay nothing for them.
template <int MODE, int BM, int BN, int WAVES_M, int WAVES_N, bool F32OUT = false, int STATS = 0, int NWRAP = 1,
          bool REMAP = false, int EPI = 0, bool GROUP = false>
__global__ void __launch_bounds__(256, ((BM / WAVES_M / 32) * (BN / WAVES_N / 32) >= 8 ? 2 : 1)) igemm_kernel(IgemmArgs a) {
  // (tiles whose accumulators take 128 registers: two waves per SIMD, i.e. two workgroups per compute unit, is what their
  // LDS allows; the bound keeps the other registers within the 128 that leaves)
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int AV = BM / 64;                  // activation vectors per thread per step
  constexpr int BV = BN >= 64 ? BN / 64 : 1;   // filter vectors per thread per step
  constexpr int BN_PAD = BN < 64 ? 64 : BN;    // filter rows in LDS (a full 64-row store pass)
  constexpr int NS = 3;                        // LDS stages: tile kt multiplies, kt+1 and kt+2 are in flight
  constexpr int STAGE = (BM + BN_PAD) * BK;    // elements per stage: activation rows, then filter rows
  constexpr int MAIN_BYTES = NS * STAGE * 2;
  constexpr int EROWS = WM < 64 ? WM : 64;     // rows staged per epilogue pass
  constexpr int EPITCH = WN + 8;
  constexpr int EPI_BYTES = 4 * EROWS * EPITCH * 2;
  constexpr int SMEM = MAIN_BYTES > EPI_BYTES ? MAIN_BYTES : EPI_BYTES;
  __shared__ __attribute__((aligned(16))) char smem[SMEM];
  bf16_t* tiles = reinterpret_cast<bf16_t*>(smem);  // [NS][BM + BN_PAD][BK]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave % WAVES_M) * WM, wn0 = (wave / WAVES_M) * WN;
  const unsigned tile = xcd_remap(blockIdx.x, gridDim.x);
  // row and element indices fit 32 bits: every operand is smaller than 2 GiB (conv_mfma_supported)
  unsigned tm = tile / (unsigned)a.ntiles, tn = tile % (unsigned)a.ntiles;
  if (GROUP) {
    // Wide outputs (a filter matrix that does not fit an L2): tiles run down groups of group_m row
    // tiles before moving to the next column tile, so that the workgroups resident at one time share
    // a few filter tiles and a few activation tiles instead of sweeping the whole filter matrix.
    const unsigned per = (unsigned)a.group_m * (unsigned)a.ntiles;
    const unsigned grp = tile / per, loc = tile - grp * per;
    const unsigned mt = (unsigned)((a.M + BM - 1) / BM);
    const unsigned gm = mt - grp * a.group_m < (unsigned)a.group_m ? mt - grp * a.group_m : (unsigned)a.group_m;
    tm = grp * a.group_m + loc % gm;
    tn = loc / gm;
  }
  const int m0 = (int)tm * BM;
  const int n0 = (int)tn * BN;
  const int M = (int)a.M;
  const rsrc_words_t rsrc = make_rsrc_words(a.src, a.src_bytes);
  const rsrc_words_t rwt = make_rsrc_words(a.wt, a.wt_bytes);

  // ---- per-thread gather state ---------------------------------------------------------------------
  // A wave's load instruction fills 16 consecutive tile rows (64 lanes x 16 bytes, in lane order), so
  // thread tid owns LDS slot tid & 3 of rows (tid >> 2) + 64 j; the slot holds the 16-byte column
  // slot ^ ((row >> 2) & 3) of the tile (see lds_off), the same for all of the thread's rows.
  const int lrow = tid >> 2;
  const int kvec = (tid & 3) ^ ((tid >> 4) & 3);
  const int P = a.src_pitch ? a.src_pitch : a.Cs;   // channels per pixel of the gathered tensor
  const int cs0 = a.sliced ? n0 : 0;                // first channel this tile gathers (sliced launches)
  int rowoff[AV];                 // element offset of (image, h0, w0, first gathered channel); may be negative
  uint32_t hmask[AV], wmask[AV];  // bit r / s set: tap row r / column s reads inside the image
#pragma unroll
  for (int j = 0; j < AV; j++) {
    const int m = m0 + lrow + 64 * j;
    const bool rowok = m < M;
    if (a.pointwise) {  // 1x1 filter, stride 1, no padding: row m of the gathered tensor, every tap inside
      hmask[j] = rowok ? 1u : 0u;
      wmask[j] = 1u;
      rowoff[j] = m * P + cs0;
      continue;
    }
    const unsigned mm = rowok ? (unsigned)m : 0u;
    const unsigned q = mm / (unsigned)a.Wd;
    const int wd = (int)(mm - q * (unsigned)a.Wd);
    const int b = (int)(q / (unsigned)a.Hd);
    const int hd = (int)(q - (unsigned)b * (unsigned)a.Hd);
    const int hh = MODE == 0 ? hd * a.stride - a.pad : hd + a.pad;
    const int ww = MODE == 0 ? wd * a.stride - a.pad_w : wd + a.pad_w;
    uint32_t hm = 0, wm = 0;
    for (int r = 0; r < a.kh; r++) {
      const int hs = MODE == 0 ? hh + r : hh - r;
      if (hs >= 0 && hs < a.Hs) hm |= 1u << r;
    }
    for (int t = 0; t < a.kw; t++) {
      const int ws = MODE == 0 ? ww + t : ww - t;
      if (ws >= 0 && ws < a.Ws) wm |= 1u << t;
    }
    hmask[j] = rowok ? hm : 0u;
    wmask[j] = wm;
    rowoff[j] = ((b * a.Hs + hh) * a.Ws + ww) * P + cs0;
  }
  uint32_t woff[BV];  // byte offset of this thread's filter row (+ its 16-byte column), ~0 if masked
#pragma unroll
  for (int j = 0; j < BV; j++) {
    const int n = n0 + lrow + 64 * j;
    woff[j] = ((lrow + 64 * j) < BN && n < a.N) ? (uint32_t)(n * a.K + kvec * 8) * 2u : 0xffffffffu;
  }
  // position of this thread's vector in the contraction: tap (kr, ks) and channel kc
  int kc = kvec * 8, kr = 0, ks = 0;
  {
    const int tap = kc / a.Cs;
    kc -= tap * a.Cs;
    kr = tap / a.kw;
    ks = tap - kr * a.kw;
  }
  const int KT = (a.K + BK - 1) / BK;
  const int tapdir = MODE == 0 ? 1 : -1;

  // LDS byte address of this wave's first 16 rows of the stage-0 activation tile
  const uint32_t lds_wave = (uint32_t)(uintptr_t)(CD_LDS char*)smem +
                            (uint32_t)__builtin_amdgcn_readfirstlane(tid >> 6) * (16u * BK * 2u);
  // Issues the loads of one step into the stage at byte offset stage_b.  Always issues them (a step at
  // or beyond the end of the contraction has every vector masked, costs no memory traffic and writes
  // zeros), so that the number of loads in flight is the same at every step, and is straight-line code.
  auto gload = [&](uint32_t stage_b, int kt) {
    const uint32_t kokb = kr < a.kh ? 1u : 0u;
    const int koff = tapdir * (kr * a.Ws + ks) * P + kc;
    const uint32_t krs = (uint32_t)kr & 31u, kss = (uint32_t)ks & 31u;
#pragma unroll
    for (int j = 0; j < AV; j++) {
      const uint32_t okb = (hmask[j] >> krs) & (wmask[j] >> kss) & kokb;
      const uint32_t off = (uint32_t)(rowoff[j] + koff) * 2u;
      load_lds16(rsrc, lds_wave + stage_b + (uint32_t)j * (64u * BK * 2u), okb ? off : 0xffffffffu);
    }
    const uint32_t wk = (uint32_t)kt * (BK * 2u);
#pragma unroll
    for (int j = 0; j < BV; j++) {
      const uint32_t off = woff[j] + wk;
      load_lds16(rwt, lds_wave + stage_b + (uint32_t)(BM + j * 64) * (BK * 2u),
                 ((kokb != 0u) & (woff[j] != 0xffffffffu)) ? off : 0xffffffffu);
    }
    // advance to the next step: NWRAP sub-steps, each crossing at most one tap boundary
#pragma unroll
    for (int u = 0; u < NWRAP; u++) {
      kc += BK / NWRAP;
      const bool wrap = kc >= a.Cs;
      kc -= wrap ? a.Cs : 0;
      ks += wrap ? 1 : 0;
      const bool wrap2 = ks == a.kw;
      ks = wrap2 ? 0 : ks;
      kr += wrap2 ? 1 : 0;
    }
  };

  // STATS 2: what the epilogue reads besides the tile itself (the BatchNorm's input and its ReLU bits at this lane's
  // output vectors) is requested now and arrives during the main loop.  (Vector memory operations retire in order:
  // the main loop's first wait also waits for these, and the compiler's own waits for them can only be too strict.)
  constexpr int BS_LPR = WN / 8, BS_RPP = 64 / BS_LPR, BS_EROWS = WM < 64 ? WM : 64;
  constexpr int BS_NV = STATS == 2 ? (WM / BS_EROWS) * (BS_EROWS / BS_RPP) : 1;
  uint4 bs_x[BS_NV];
  uint32_t bs_bits[BS_NV];
  if (STATS == 2) {
    const int er_ = lane / BS_LPR, n = n0 + wn0 + (lane % BS_LPR) * 8;
#pragma unroll
    for (int v = 0; v < BS_NV; v++) {
      const int pass = v / (BS_EROWS / BS_RPP), pp = v % (BS_EROWS / BS_RPP);
      const int m = m0 + wm0 + pass * BS_EROWS + pp * BS_RPP + er_;
      bs_x[v] = make_uint4(0, 0, 0, 0);
      bs_bits[v] = 0u;
      if (m < M && n < a.N) {
        const unsigned idx = (unsigned)m * (unsigned)a.N + (unsigned)n;
        bs_x[v] = *reinterpret_cast<const uint4*>(a.bn_x + idx);
        bs_bits[v] = a.bn_mask ? a.bn_mask[idx >> 3] : 0xffu;
      }
    }
  }
  f32x16_t acc[TN][TM];
#pragma unroll
  for (int i = 0; i < TN; i++)
#pragma unroll
    for (int j = 0; j < TM; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  const int frow = lane & 31, fcv = lane >> 5;
  bf16x8_t wf[2][TN], xf[2][TM];  // [k16 half][tile]
  auto read_frags = [&](uint32_t stage_e) {
#pragma unroll
    for (int kk = 0; kk < 2; kk++) {
#pragma unroll
      for (int i = 0; i < TN; i++)
        wf[kk][i] = *reinterpret_cast<const bf16x8_t*>(tiles + stage_e + BM * BK + lds_off(wn0 + i * 32 + frow, kk * 2 + fcv));
#pragma unroll
      for (int j = 0; j < TM; j++)
        xf[kk][j] = *reinterpret_cast<const bf16x8_t*>(tiles + stage_e + lds_off(wm0 + j * 32 + frow, kk * 2 + fcv));
    }
  };
  auto mfma_step = [&]() {
#pragma unroll
    for (int kk = 0; kk < 2; kk++)
#pragma unroll
      for (int i = 0; i < TN; i++)
#pragma unroll
        for (int j = 0; j < TM; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[kk][i], xf[kk][j], acc[i][j], 0, 0, 0);
  };
  // Three stages rotate: at step kt the stage `cur` holds tile kt, `nxt` receives tile kt+1 (loads issued
  // one step ago) and `fre` (read last at step kt-1) receives tile kt+2.  One barrier per step: it
  // publishes tile kt (every wave has waited for its own loads of it) and retires the reads of tile kt-1.
  uint32_t cur = 0, nxt = STAGE, fre = 2 * STAGE;  // element offsets
  gload(cur * 2u, 0);
  gload(nxt * 2u, 1);
  for (int kt = 0; kt < KT; kt++) {
    wait_vmem<AV + BV>();   // all but the newest step's loads have landed
    __syncthreads();
    gload(fre * 2u, kt + 2);
    read_frags(cur);
    mfma_step();
    const uint32_t t = cur; cur = nxt; nxt = fre; fre = t;
  }
  wait_vmem<0>();  // the masked loads past the end still write (zeros) into the stages the epilogue reuses

  // accumulator layout: lane holds pixel column (lane % 32); register v holds channel
  // 8*(v/4) + 4*(lane/32) + v%4 of the 32x32 tile
  // per-column bias: register v of tile i belongs to channel n0 + wn0 + 32 i + 8 (v / 4) + 4 (lane / 32) + v % 4
  if (EPI >= 1) {
#pragma unroll
    for (int i = 0; i < TN; i++)
#pragma unroll
      for (int g = 0; g < 4; g++) {
        const int n = n0 + wn0 + i * 32 + 8 * g + 4 * (lane >> 5);
        float bv[4];
#pragma unroll
        for (int q = 0; q < 4; q++) bv[q] = n + q < a.N ? bf16_to_f32(a.bias[n + q]) : 0.f;
#pragma unroll
        for (int j = 0; j < TM; j++)
#pragma unroll
          for (int q = 0; q < 4; q++) acc[i][j][4 * g + q] += bv[q];
      }
  }
  if (F32OUT) {
    // one 32-row tile row of the wave at a time: [32][WN] floats (+4 of padding) per wave
    constexpr int FP = WN + 4;
    static_assert(4 * 32 * FP * 4 <= SMEM, "fp32 staging fits the tile memory");
    float* fst = reinterpret_cast<float*>(smem) + wave * 32 * FP;
    float* dst = reinterpret_cast<float*>(a.dst);
    constexpr int FLPR = WN / 4;       // lanes per output row (16-byte vectors)
    constexpr int FRPP = 64 / FLPR;    // rows per store instruction
    const int fr = lane / FLPR, fc = (lane % FLPR) * 4;
    __syncthreads();  // the main loop's tiles are no longer read
#pragma unroll
    for (int j = 0; j < TM; j++) {
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int i = 0; i < TN; i++)
#pragma unroll
        for (int g = 0; g < 4; g++)
          *reinterpret_cast<float4*>(fst + frow * FP + i * 32 + 8 * g + 4 * (lane >> 5)) =
              make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int p = 0; p < 32 / FRPP; p++) {
        const int row = p * FRPP + fr;
        const int m = m0 + wm0 + j * 32 + row;
        const int n = n0 + wn0 + fc;
        if (m < M && n < a.N) {
          const float4 v = *reinterpret_cast<const float4*>(fst + row * FP + fc);
          float* dp = dst + ((int64_t)m * a.N + n);
          if (n + 3 < a.N && (a.N & 3) == 0) {
            *reinterpret_cast<float4*>(dp) = v;
          } else {  // ragged or unaligned row ends
            const float e[4] = {v.x, v.y, v.z, v.w};
            for (int q = 0; q < 4 && n + q < a.N; q++) dp[q] = e[q];
          }
        }
      }
    }
    return;
  }
  if (EPI == 2) {
#pragma unroll
    for (int i = 0; i < TN; i++)
#pragma unroll
      for (int j = 0; j < TM; j++)
#pragma unroll
        for (int v = 0; v < 16; v++) acc[i][j][v] = fmaxf(acc[i][j][v], 0.f);
  }
  // ---- epilogue: fp32 -> bf16, transpose through LDS, 16-byte stores along the channels -------------
  bf16_t* stage = reinterpret_cast<bf16_t*>(smem) + wave * EROWS * EPITCH;
  constexpr int LPR = WN / 8;        // lanes per output row
  constexpr int RPP = 64 / LPR;      // rows per pass
  constexpr int TPG = EROWS / 32;    // 32-row tiles per staging pass
  const int er = lane / LPR, ec = (lane % LPR) * 8;
  // STATS: per-wave column sums [WAVES_M][2][BN], behind the staging rows
  static_assert(STATS == 0 || EPI_BYTES + WAVES_M * 2 * BN * 4 <= SMEM, "no room for the column sums behind the staging rows");
  static_assert(STATS != 2 || !REMAP, "the backward sums are taken where the rows are stored in order");
  // STATS 2: running sums of dz and of dz * x over this lane's 8 channels (the same in every pass); the mean and the
  // scale of xhat = (x - mean) * invstd are applied to the tile's sums at the end (the sums are linear in x)
  float bs0[8], bs1[8];
  if (STATS == 2) {
#pragma unroll
    for (int k = 0; k < 8; k++) { bs0[k] = 0.f; bs1[k] = 0.f; }
  }
  float* red = reinterpret_cast<float*>(smem + EPI_BYTES);
  __syncthreads();  // the main loop's tiles are no longer read: the staging rows alias them
#pragma unroll
  for (int g0 = 0; g0 < TM; g0 += TPG) {
    // The staging rows belong to this wave alone, and a wave's LDS accesses execute in program order:
    // no block barrier between its writes, its reads and the next pass's writes.
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int i = 0; i < TN; i++)
#pragma unroll
      for (int j = 0; j < TPG; j++)
#pragma unroll
        for (int g = 0; g < 4; g++) {
          uint2 p;
          p.x = pack_bf16x2(acc[i][g0 + j][4 * g + 0], acc[i][g0 + j][4 * g + 1]);
          p.y = pack_bf16x2(acc[i][g0 + j][4 * g + 2], acc[i][g0 + j][4 * g + 3]);
          *reinterpret_cast<uint2*>(stage + (j * 32 + frow) * EPITCH + i * 32 + 8 * g + 4 * (lane >> 5)) = p;
        }
    __builtin_amdgcn_wave_barrier();
    if (STATS == 1) {
      // Column sums and sums of squares of the staged (rounded) rows on the matrix cores, which idle in
      // the epilogue: the transposing LDS read hands a lane 8 pixels of its column (16 pixels x 32
      // columns per fragment, the operand layout of wgrad_kernel); ones^T Y gives the sums in every row
      // of one accumulator tile, Y^T Y the sums of squares on the diagonal of another.  Rows past M and
      // columns past N were computed from zero-filled operands and add nothing.
      const int grp = lane >> 4, li = lane & 15;
      const int tr_m = 8 * (grp >> 1) + (li >> 2), tr_c = 16 * (grp & 1) + 4 * (li & 3);
      const __bf16 one = (__bf16)1.0f;
      const bf16x8_t ones = {one, one, one, one, one, one, one, one};
      const int wmi = wave % WAVES_M, c = lane & 31;
#pragma unroll 1
      for (int i = 0; i < TN; i++) {   // one 32-column block at a time: two accumulator tiles live
        f32x16_t ds, dq;
#pragma unroll
        for (int v = 0; v < 16; v++) { ds[v] = 0.f; dq[v] = 0.f; }
#pragma unroll
        for (int pc = 0; pc < EROWS / 16; pc++) {
          const bf16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
              (CD_LDS bf16x4_t*)(stage + (pc * 16 + tr_m) * EPITCH + i * 32 + tr_c));
          const bf16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
              (CD_LDS bf16x4_t*)(stage + (pc * 16 + tr_m + 4) * EPITCH + i * 32 + tr_c));
          const bf16x8_t f = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
          ds = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, f, ds, 0, 0, 0);
          dq = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, f, dq, 0, 0, 0);
        }
        // every lane holds the sum of its column, one half-wave per column the sum of squares; a later
        // pass over further rows of the tile adds to what this lane wrote
        float* r0 = red + (wmi * 2 + 0) * BN + wn0 + i * 32 + c;
        float* r1 = red + (wmi * 2 + 1) * BN + wn0 + i * 32 + c;
        const float sq = tile_diagonal(dq, c);
        if (lane < 32) *r0 = g0 == 0 ? ds[0] : *r0 + ds[0];
        if (((c >> 2) & 1) == (lane >> 5)) *r1 = g0 == 0 ? sq : *r1 + sq;
      }
    }
#pragma unroll
    for (int p = 0; p < EROWS / RPP; p++) {
      const int row = p * RPP + er;
      int m = m0 + wm0 + g0 * 32 + row;
      const int n = n0 + wn0 + ec;
      if (m < M && n < a.N) {
        uint4 v = *reinterpret_cast<const uint4*>(stage + row * EPITCH + ec);
        if (REMAP) {  // strided placement of the rows (parity class of a stride-2 dgrad)
          const unsigned q = (unsigned)m / (unsigned)a.Wd;
          const int wd = m - (int)(q * (unsigned)a.Wd);
          const int b = (int)(q / (unsigned)a.Hd);
          const int hd = (int)q - b * a.Hd;
          m = (b * a.Ho + hd * a.omul + a.ooff_h) * a.Wo + wd * a.omul + a.ooff_w;
        }
        const unsigned idx = (unsigned)m * (unsigned)a.N + (unsigned)n;
        bf16_t* dp = a.dst + idx;
        if (a.accumulate) {
          const uint4 o = *reinterpret_cast<const uint4*>(a.addend ? a.addend + idx : dp);
          const uint32_t vv[4] = {v.x, v.y, v.z, v.w};
          uint32_t oo[4] = {o.x, o.y, o.z, o.w};
          if (a.addend_gate) {
            const uint32_t bits = a.addend_gate[idx >> 3];
#pragma unroll
            for (int q = 0; q < 4; q++)
              oo[q] &= ((bits >> (2 * q)) & 1u ? 0x0000ffffu : 0u) | ((bits >> (2 * q + 1)) & 1u ? 0xffff0000u : 0u);
          }
          uint32_t r[4];
#pragma unroll
          for (int q = 0; q < 4; q++)
            r[q] = pack_bf16x2(__uint_as_float(vv[q] << 16) + __uint_as_float(oo[q] << 16),
                               __uint_as_float(vv[q] & 0xffff0000u) + __uint_as_float(oo[q] & 0xffff0000u));
          v = make_uint4(r[0], r[1], r[2], r[3]);
        }
        if (a.relu_out) {
          const uint4 y = *reinterpret_cast<const uint4*>(a.relu_out + idx);
          const uint32_t yy[4] = {y.x, y.y, y.z, y.w};
          uint32_t vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
          for (int q = 0; q < 4; q++)   // a bf16 is positive iff its bits, read as int16, are
            vv[q] &= ((int16_t)(yy[q] & 0xffffu) > 0 ? 0x0000ffffu : 0u) | ((int16_t)(yy[q] >> 16) > 0 ? 0xffff0000u : 0u);
          v = make_uint4(vv[0], vv[1], vv[2], vv[3]);
        }
        if (STATS == 2) {   // the stored values feed the sums of the BatchNorm's backward pass
          const uint4 xr = bs_x[(g0 / TPG) * (EROWS / RPP) + p];
          const uint32_t bits = bs_bits[(g0 / TPG) * (EROWS / RPP) + p];
          const uint32_t gv[4] = {v.x, v.y, v.z, v.w}, xv[4] = {xr.x, xr.y, xr.z, xr.w};
#pragma unroll
          for (int q = 0; q < 4; q++) {
            const float d0 = (bits >> (2 * q)) & 1u ? __uint_as_float(gv[q] << 16) : 0.f;
            const float d1 = (bits >> (2 * q + 1)) & 1u ? __uint_as_float(gv[q] & 0xffff0000u) : 0.f;
            bs0[2 * q] += d0;
            bs0[2 * q + 1] += d1;
            bs1[2 * q] += d0 * __uint_as_float(xv[q] << 16);
            bs1[2 * q + 1] += d1 * __uint_as_float(xv[q] & 0xffff0000u);
          }
        }
        *reinterpret_cast<uint4*>(dp) = v;
      }
    }
  }
  if (STATS == 2) {
    // lanes that share their 8 channels (one per row of a pass) add up, the first of them hands the wave's sums over
#pragma unroll
    for (int k = 0; k < 8; k++) {
#pragma unroll
      for (int off = LPR; off < 64; off <<= 1) {
        bs0[k] += __shfl_xor(bs0[k], off, 64);
        bs1[k] += __shfl_xor(bs1[k], off, 64);
      }
    }
    if (lane < LPR) {
      const int wmi = wave % WAVES_M;
#pragma unroll
      for (int k = 0; k < 8; k++) {
        red[(wmi * 2 + 0) * BN + wn0 + ec + k] = bs0[k];
        red[(wmi * 2 + 1) * BN + wn0 + ec + k] = bs1[k];
      }
    }
  }
  if (STATS) {
    // fold the waves of a column
    __syncthreads();
    if (tid < BN && n0 + tid < a.N) {
      float s0 = 0.f, s1 = 0.f;
#pragma unroll
      for (int w = 0; w < WAVES_M; w++) { s0 += red[(w * 2 + 0) * BN + tid]; s1 += red[(w * 2 + 1) * BN + tid]; }
      if (STATS == 2) s1 = (s1 - a.bn_stats[n0 + tid] * s0) * a.bn_stats[a.N + n0 + tid];   // sum dz x -> sum dz xhat
      const int64_t mt = tm;
      a.stat_partials[mt * stat_pitch(a.N) + n0 + tid] = s0;
      a.stat_partials[mt * stat_pitch(a.N) + a.N + n0 + tid] = s1;
    }
  }
}

// Output tile of the wide-output kernels (N > 64): 128x128 (three workgroups per compute unit, 768 at a
// time), 256x128 or 128x256 (two per compute unit, 512 at a time).  Measured on the layer shapes of
// ResNet-50 at batch 256:
//  - a short contraction leaves a tile little more than its prologue and epilogue, and the larger
//    tiles halve those per output element: 128x256, which also reads the activations once per 256
//    columns and stores 512-byte row segments, wins up to K = 1024; with very short contractions
//    onto many columns (K <= 128, N >= 512) 256x128 wins instead;
//  - otherwise the taller tile pays only when its last round of workgroups is clearly fuller.
enum { TILE_SQUARE = 0, TILE_TALL = 1, TILE_WIDE = 2 };
static int igemm_tile(int64_t M, int N, int K) {
  if (N <= 64) return TILE_SQUARE;
  if (g_tune_tile == 2) return TILE_SQUARE;
  if (g_tune_tile == 3) return TILE_TALL;
  if (g_tune_tile == 4) return N % 256 == 0 ? TILE_WIDE : TILE_SQUARE;
  if (K <= 128 && N >= 512) return TILE_TALL;
  if (N % 256 == 0 && K <= 1024) return TILE_WIDE;
  const int64_t t128 = cdiv(M, 128) * cdiv(N, 128), t256 = cdiv(M, 256) * cdiv(N, 128);
  const double e128 = (double)t128 / (double)(cdiv(t128, 768) * 768), e256 = (double)t256 / (double)(cdiv(t256, 512) * 512);
  return e256 > 1.2 * e128 ? TILE_TALL : TILE_SQUARE;
}
int conv_fprop_tile_class(const ConvGeom& g, bool bias) {
  if (g.Cout <= 64) return 2;
  if (g.Cin < BK || bias) return 0;
  const int t = igemm_tile(g.M(), g.Cout, (int)g.K());
  return t == TILE_SQUARE ? 0 : (t == TILE_WIDE ? 1 : 2);
}

// returns the number of m-tiles (= statistics chunks when STATS)
template <int MODE, int STATS, int NWRAP, bool REMAP, int EPI>
static int launch_igemm_w(IgemmArgs a, hipStream_t s) {
  a.pointwise = (a.kh == 1 && a.kw == 1 && a.stride == 1 && a.pad == 0 && a.pad_w == 0 && a.Hs == a.Hd &&
                 a.Ws == a.Wd) ? 1 : 0;
  a.group_m = 1;
  const int tile = (NWRAP == 1 && !REMAP && EPI == 0 && !a.sliced) ? igemm_tile(a.M, a.N, a.K) : TILE_SQUARE;
  if (tile == TILE_TALL) {
    a.ntiles = (int)cdiv(a.N, 128);
    const int mt = (int)cdiv(a.M, 256);
    hipLaunchKernelGGL((igemm_kernel<MODE, 256, 128, 2, 2, false, STATS, 1, false>),
                       dim3((unsigned)((int64_t)mt * a.ntiles)), dim3(256), 0, s, a);
    return mt;
  }
  if (tile == TILE_WIDE) {
    a.ntiles = a.N / 256;
    const int mt = (int)cdiv(a.M, 128);
    hipLaunchKernelGGL((igemm_kernel<MODE, 128, 256, 2, 2, false, STATS, 1, false>),
                       dim3((unsigned)((int64_t)mt * a.ntiles)), dim3(256), 0, s, a);
    return mt;
  }
  if (a.N > 64 && g_tune_tile != 1 && !a.sliced) {
    a.ntiles = (int)cdiv(a.N, 128);
    const int mt = (int)cdiv(a.M, 128);
    hipLaunchKernelGGL((igemm_kernel<MODE, 128, 128, 2, 2, false, STATS, NWRAP, REMAP, EPI>),
                       dim3((unsigned)((int64_t)mt * a.ntiles)), dim3(256), 0, s, a);
    return mt;
  }
  if (a.sliced) {   // grouped convolution: one column tile per slice of Cs = 32 or 64 channels
    a.ntiles = a.N / a.Cs;
    const int mt = (int)cdiv(a.M, 256);
    const dim3 grid((unsigned)((int64_t)mt * a.ntiles));
    if (a.Cs == 64) hipLaunchKernelGGL((igemm_kernel<MODE, 256, 64, 4, 1, false, STATS, NWRAP, REMAP, EPI>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((igemm_kernel<MODE, 256, 32, 4, 1, false, STATS, NWRAP, REMAP, EPI>), grid, dim3(256), 0, s, a);
    return mt;
  }
  a.ntiles = (int)cdiv(a.N, 64);
  const int mt = (int)cdiv(a.M, 256);
  if (a.N > 32)
    hipLaunchKernelGGL((igemm_kernel<MODE, 256, 64, 4, 1, false, STATS, NWRAP, REMAP, EPI>),
                       dim3((unsigned)((int64_t)mt * a.ntiles)), dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL((igemm_kernel<MODE, 256, 32, 4, 1, false, STATS, NWRAP, REMAP, EPI>), dim3((unsigned)mt), dim3(256),
                       0, s, a);
  return mt;
}
template <int MODE, int STATS, bool REMAP = false, int EPI = 0>
static int launch_igemm(IgemmArgs a, hipStream_t s) {
  return a.Cs >= BK ? launch_igemm_w<MODE, STATS, 1, REMAP, EPI>(a, s) : launch_igemm_w<MODE, STATS, 4, REMAP, EPI>(a, s);
}

bool conv_mfma_supported(const ConvGeom& g) {
  // 32-bit byte offsets into every operand, tap masks of at most 32 bits
  const int64_t lim = 1LL << 31;
  return g.Cin % 8 == 0 && g.Cout % 8 == 0 && (g.stride == 1 || g.stride == 2) && g.kh == g.kw && g.kh <= 7 &&
         g.B * g.H * g.W * (int64_t)g.Cin * 2 < lim && g.M() * (int64_t)g.Cout * 2 < lim &&
         (int64_t)g.Cout * g.K() * 2 < lim;
}

void linear_fwd_mfma(const bf16_t* x, const bf16_t* w, const bf16_t* bias, float* y, int64_t B, int F, int C,
                     hipStream_t s) {
  IgemmArgs a;
  a.src = x; a.wt = w; a.dst = reinterpret_cast<bf16_t*>(y); a.bias = bias; a.stat_partials = nullptr;
  a.M = B; a.N = C; a.K = F;
  a.Hs = 1; a.Ws = 1; a.Cs = F; a.Hd = 1; a.Wd = 1; a.kh = 1; a.kw = 1; a.stride = 1; a.pad = 0; a.pad_w = 0;
  a.omul = 0; a.ooff_h = a.ooff_w = 0; a.Ho = a.Wo = 1;
  a.accumulate = 0;
  a.pointwise = 1;
  a.group_m = 8;
  a.src_bytes = (uint32_t)(B * (int64_t)F * 2);
  a.wt_bytes = (uint32_t)((int64_t)C * F * 2);
  a.ntiles = (int)cdiv(C, 128);
  const dim3 grid((unsigned)(cdiv(B, 128) * a.ntiles));
  // a filter matrix beyond an L2's 4 MiB under a wide output: grouped tile order
  const bool group = (int64_t)C * F * 2 > (4 << 20) && C >= 2048;
  if (group) {
    if (bias) hipLaunchKernelGGL((igemm_kernel<0, 128, 128, 2, 2, true, false, 1, false, 1, true>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((igemm_kernel<0, 128, 128, 2, 2, true, false, 1, false, 0, true>), grid, dim3(256), 0, s, a);
  } else {
    if (bias) hipLaunchKernelGGL((igemm_kernel<0, 128, 128, 2, 2, true, false, 1, false, 1, false>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((igemm_kernel<0, 128, 128, 2, 2, true, false, 1, false, 0, false>), grid, dim3(256), 0, s, a);
  }
}

int conv_fprop_mfma(const bf16_t* x, const bf16_t* w, const bf16_t* bias, bool relu, bf16_t* y, const ConvGeom& g,
                    float* stat_partials, hipStream_t s) {
  IgemmArgs a;
  a.bias = bias;
  a.stat_partials = stat_partials;
  a.src = x; a.wt = w; a.dst = y;
  a.M = g.M(); a.N = g.Cout; a.K = g.K();
  a.Hs = g.H; a.Ws = g.W; a.Cs = g.Cin; a.Hd = g.Ho; a.Wd = g.Wo;
  a.kh = g.kh; a.kw = g.kw; a.stride = g.stride; a.pad = g.pad; a.pad_w = g.pad;
  a.omul = 0; a.ooff_h = a.ooff_w = 0; a.Ho = g.Ho; a.Wo = g.Wo;
  a.accumulate = 0; a.ntiles = 1;
  a.src_bytes = (uint32_t)(g.B * g.H * g.W * (int64_t)g.Cin * 2);
  a.wt_bytes = (uint32_t)((int64_t)g.Cout * g.K() * 2);
  if (bias) {  // bias (+ ReLU) in the epilogue; no statistics variant (a BatchNorm follows bias-free convolutions)
    if (stat_partials) return -1;
    return relu ? launch_igemm<0, false, false, 2>(a, s) : launch_igemm<0, false, false, 1>(a, s);
  }
  if (relu) return -1;  // ReLU without bias does not occur in the supported graphs
  return stat_partials ? launch_igemm<0, true>(a, s) : launch_igemm<0, false>(a, s);
}

// w[Cout][kh][kw][Cin] -> wt[Cin][th][tw][Cout] with filter row r = r0 - 2*jh, column s = s0 - 2*jw
__global__ void __launch_bounds__(256) gather_weight_class_k(const bf16_t* __restrict__ w, bf16_t* __restrict__ wt,
                                                             int cout, int kh, int kw, int cin, int th, int tw, int r0,
                                                             int s0) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)cin * th * tw * cout) return;
  const int n = i % cout;
  int64_t q = i / cout;
  const int jw = q % tw; q /= tw;
  const int jh = q % th;
  const int c = q / th;
  wt[i] = w[(((int64_t)n * kh + (r0 - 2 * jh)) * kw + (s0 - 2 * jw)) * cin + c];
}

__global__ void __launch_bounds__(256) fill_zero16_k(uint4* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = make_uint4(0, 0, 0, 0);
}

// ---- filter re-layouts of many data gradients in one launch ------------------------------------------------------
constexpr int kLayoutJobs = 48;   // jobs per launch: the table travels in the kernel arguments
struct LayoutBatch { WeightLayoutJob j[kLayoutJobs]; int n; int64_t total; };
__global__ void __launch_bounds__(256) relayout_weights_k(LayoutBatch b) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= b.total) return;
  int k = 0;
  while (k + 1 < b.n && b.j[k + 1].first <= i) k++;
  const WeightLayoutJob& q = b.j[k];
  const int64_t e = i - q.first;
  const int n = (int)(e % q.cout);
  int64_t t = e / q.cout;
  const int jw = (int)(t % q.tw); t /= q.tw;
  const int jh = (int)(t % q.th);
  const int c = (int)(t / q.th);
  q.wt[e] = q.w[(((int64_t)n * q.kh + (q.r0 + q.rstep * jh)) * q.kw + (q.s0 + q.rstep * jw)) * q.cin + c];
}
void relayout_weights_batch(std::vector<WeightLayoutJob>& jobs, hipStream_t s) {
  for (size_t j0 = 0; j0 < jobs.size(); j0 += kLayoutJobs) {
    LayoutBatch b;
    b.n = (int)std::min<size_t>(kLayoutJobs, jobs.size() - j0);
    b.total = 0;
    for (int k = 0; k < b.n; k++) {
      WeightLayoutJob& q = jobs[j0 + k];
      q.first = b.total;
      b.j[k] = q;
      b.total += (int64_t)q.cin * q.th * q.tw * q.cout;
    }
    if (b.total > 0)
      hipLaunchKernelGGL(relayout_weights_k, dim3((unsigned)cdiv(b.total, 256)), dim3(256), 0, s, b);
  }
}
// The parity classes of a stride-2 data gradient (see conv_dgrad_mfma): calls f(ph, pw, th, tw, tminh, tminw) for every
// class that has taps and pixels.
template <typename F>
static void for_each_parity_class(const ConvGeom& g, F f) {
  for (int ph = 0; ph < 2; ph++)
    for (int pw = 0; pw < 2; pw++) {
      const int loh = ph + g.pad - g.kh + 1, low = pw + g.pad - g.kw + 1;
      const int tminh = loh <= 0 ? -((-loh) >> 1) : (loh + 1) >> 1, tmaxh = (ph + g.pad) >> 1;
      const int tminw = low <= 0 ? -((-low) >> 1) : (low + 1) >> 1, tmaxw = (pw + g.pad) >> 1;
      const int th = tmaxh - tminh + 1, tw = tmaxw - tminw + 1;
      const int hd = (g.H - ph + 1) / 2, wd = (g.W - pw + 1) / 2;
      if (th <= 0 || tw <= 0 || hd <= 0 || wd <= 0) continue;
      f(ph, pw, th, tw, tminh, tminw);
    }
}
int64_t conv_dgrad_layout_elems(const ConvGeom& g) {
  if (g.stride == 1) return (int64_t)g.Cout * g.K();
  int64_t n = 0;
  for_each_parity_class(g, [&](int, int, int th, int tw, int, int) { n += ((int64_t)g.Cin * th * tw * g.Cout + 7) / 8 * 8; });
  return n;
}
void conv_dgrad_layout_jobs(const bf16_t* w, bf16_t* wt, const ConvGeom& g, std::vector<WeightLayoutJob>& jobs) {
  if (g.stride == 1) {   // wt[Cin][kh][kw][Cout] = w[Cout][kh][kw][Cin]
    jobs.push_back(WeightLayoutJob{w, wt, g.Cout, g.kh, g.kw, g.Cin, g.kh, g.kw, 0, 0, 1, 0});
    return;
  }
  int64_t woff = 0;
  for_each_parity_class(g, [&](int ph, int pw, int th, int tw, int tminh, int tminw) {
    jobs.push_back(WeightLayoutJob{w, wt + woff, g.Cout, g.kh, g.kw, g.Cin, th, tw, ph + g.pad - 2 * tminh, pw + g.pad - 2 * tminw,
                                   -2, 0});
    woff += ((int64_t)g.Cin * th * tw * g.Cout + 7) / 8 * 8;
  });
}

int conv_dgrad_mfma(const bf16_t* dy, const bf16_t* w, bf16_t* wt, bf16_t* dx, const ConvGeom& g, bool accumulate,
                    hipStream_t s, const bf16_t* addend, const uint8_t* addend_gate, const bf16_t* relu_out,
                    const BnBackwardSums* bn, bool wt_ready) {
  IgemmArgs a;
  a.bias = nullptr;
  a.stat_partials = nullptr;
  a.src = dy; a.dst = dx;
  a.N = g.Cin;
  a.Hs = g.Ho; a.Ws = g.Wo; a.Cs = g.Cout;
  a.ntiles = 1;
  a.src_bytes = (uint32_t)(g.M() * (int64_t)g.Cout * 2);
  a.Ho = g.H; a.Wo = g.W;
  if (g.stride == 1) {
    if (!wt_ready) transpose_weight(w, wt, g.Cout, g.kh * g.kw, g.Cin, s);
    a.wt = wt;
    a.M = g.B * g.H * g.W; a.K = g.kh * g.kw * g.Cout;
    a.Hd = g.H; a.Wd = g.W;
    a.kh = g.kh; a.kw = g.kw; a.stride = 1; a.pad = g.pad; a.pad_w = g.pad;
    a.omul = 0; a.ooff_h = a.ooff_w = 0;
    a.accumulate = (accumulate || addend) ? 1 : 0;
    a.addend = addend;          // stride 1 only (see the declaration); never together with accumulate
    a.addend_gate = addend_gate;
    a.relu_out = relu_out;      // stride 1 only, like the addend
    a.wt_bytes = (uint32_t)((int64_t)g.Cout * g.K() * 2);
    if (bn) {
      a.bn_x = bn->x; a.bn_mask = bn->mask; a.bn_stats = bn->stats; a.stat_partials = bn->partials;
      return launch_igemm<1, 2>(a, s);
    }
    launch_igemm<1, 0>(a, s);
    return 0;
  }
  // Stride 2: input pixel (h, w) receives dy[(h + pad - r)/2, (w + pad - s)/2] * w[., r, s, .] for the taps
  // of matching parity only.  Per parity class (h%2, w%2) that is a stride-1 gather over the half
  // resolution grid h = 2h' + ph with window rows t in [tmin, tmax], ho = h' + t, r = ph + pad - 2t: a
  // MODE 0 problem with its own filter layout, writing every second row / column of dx.
  bool covered_all = true;
  for (int ph = 0; ph < 2; ph++) {
    const int tmax = (ph + g.pad) >> 1, lo = ph + g.pad - g.kh + 1;
    if (tmax < (lo <= 0 ? -((-lo) >> 1) : (lo + 1) >> 1)) covered_all = false;
  }
  if (!accumulate && !covered_all) {
    const int64_t n16 = g.B * g.H * g.W * (int64_t)g.Cin / 8;
    hipLaunchKernelGGL(fill_zero16_k, dim3((unsigned)cdiv(n16, 256)), dim3(256), 0, s, reinterpret_cast<uint4*>(dx), n16);
    accumulate = true;
  }
  int64_t woff = 0;
  for (int ph = 0; ph < 2; ph++)
    for (int pw = 0; pw < 2; pw++) {
      const int loh = ph + g.pad - g.kh + 1, low = pw + g.pad - g.kw + 1;
      const int tminh = loh <= 0 ? -((-loh) >> 1) : (loh + 1) >> 1, tmaxh = (ph + g.pad) >> 1;
      const int tminw = low <= 0 ? -((-low) >> 1) : (low + 1) >> 1, tmaxw = (pw + g.pad) >> 1;
      const int th = tmaxh - tminh + 1, tw = tmaxw - tminw + 1;
      const int hd = (g.H - ph + 1) / 2, wd = (g.W - pw + 1) / 2;
      if (th <= 0 || tw <= 0 || hd <= 0 || wd <= 0) continue;
      bf16_t* wc = wt + woff;
      const int64_t wn = (int64_t)g.Cin * th * tw * g.Cout;
      if (!wt_ready)
        hipLaunchKernelGGL(gather_weight_class_k, dim3((unsigned)cdiv(wn, 256)), dim3(256), 0, s, w, wc, g.Cout, g.kh,
                           g.kw, g.Cin, th, tw, ph + g.pad - 2 * tminh, pw + g.pad - 2 * tminw);
      woff += (wn + 7) / 8 * 8;
      a.wt = wc;
      a.M = g.B * hd * wd; a.K = th * tw * g.Cout;
      a.Hd = hd; a.Wd = wd;
      a.kh = th; a.kw = tw; a.stride = 1; a.pad = -tminh; a.pad_w = -tminw;
      a.omul = 2; a.ooff_h = ph; a.ooff_w = pw;
      a.accumulate = accumulate ? 1 : 0;
      a.wt_bytes = (uint32_t)(wn * 2);
      launch_igemm<0, 0, true>(a, s);
    }
  return 0;
}

// ---- grouped convolutions (Cin = Cout = C, groups of cg = C / groups channels) as sliced launches ----------------
// The channels are cut into slices of SW = 32 or 64 (whole groups).  Column tile s of a launch computes the SW output
// channels of slice s from the SW input channels of the same slice, read in place from the row-major tensor (pitch C),
// with a filter whose rows hold kh * kw * SW elements, zero outside the row's own group: for cg = SW the contraction
// runs over the group's channels only, for smaller groups it spends SW / cg times the grouped arithmetic on zeros.
int grouped_mfma_slice(int C, int groups) {
  if (groups < 1 || C % groups) return 0;
  const int cg = C / groups;
  const int sw = cg > 32 ? 64 : 32;
  return (C % sw == 0 && sw % cg == 0) ? sw : 0;
}

// w [C][taps][cg] -> wd [C][th * tw][SW]: row o, tap (jh, jw), column i holds w[o][r][t][i - its group's first channel
// in the slice] if input channel i of o's slice belongs to o's group, else 0; r = r0 + rstep * jh, t = s0 + rstep * jw.
// TRANSPOSED: wd [C][th * tw][SW] indexed [input channel c][tap][output channel of c's slice] (data gradients).
template <bool TRANSPOSED>
__global__ void __launch_bounds__(256) expand_sliced_weights_k(const bf16_t* __restrict__ w, bf16_t* __restrict__ wd, int C,
                                                               int kh, int kw, int cg, int SW, int th, int tw, int r0, int s0,
                                                               int rstep) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)C * th * tw * SW) return;
  const int col = (int)(idx % SW);
  const int t = (int)((idx / SW) % (th * tw));
  const int row = (int)(idx / ((int64_t)SW * th * tw));
  const int slice0 = row / SW * SW;
  const int o = TRANSPOSED ? slice0 + col : row;      // output channel
  const int ci = TRANSPOSED ? row : slice0 + col;     // input channel
  const int r = r0 + rstep * (t / tw), q = s0 + rstep * (t % tw);
  const bool ok = o / cg == ci / cg && r >= 0 && r < kh && q >= 0 && q < kw;
  wd[idx] = ok ? w[(((int64_t)o * kh + r) * kw + q) * cg + ci % cg] : (bf16_t)0;
}

static void fill_sliced(IgemmArgs& a, int C, int SW) {
  a.N = C; a.Cs = SW; a.src_pitch = C; a.sliced = 1;
  a.bias = nullptr; a.addend = nullptr; a.addend_gate = nullptr; a.relu_out = nullptr;
  a.omul = 0; a.ooff_h = a.ooff_w = 0;
  a.accumulate = 0; a.ntiles = 1;
}

int conv_grouped_fprop_mfma(const bf16_t* x, const bf16_t* w, bf16_t* wd, bf16_t* y, const ConvGeom& g, int groups,
                            float* stat_partials, hipStream_t s) {
  const int C = g.Cin, cg = C / groups, SW = grouped_mfma_slice(C, groups), taps = g.kh * g.kw;
  const int64_t nw = (int64_t)C * taps * SW;
  hipLaunchKernelGGL(expand_sliced_weights_k<false>, dim3((unsigned)cdiv(nw, 256)), dim3(256), 0, s, w, wd, C, g.kh, g.kw, cg, SW,
                     g.kh, g.kw, 0, 0, 1);
  IgemmArgs a;
  fill_sliced(a, C, SW);
  a.stat_partials = stat_partials;
  a.src = x; a.wt = wd; a.dst = y;
  a.M = g.M(); a.K = taps * SW;
  a.Hs = g.H; a.Ws = g.W; a.Hd = g.Ho; a.Wd = g.Wo;
  a.kh = g.kh; a.kw = g.kw; a.stride = g.stride; a.pad = g.pad; a.pad_w = g.pad;
  a.Ho = g.Ho; a.Wo = g.Wo;
  a.src_bytes = (uint32_t)(g.B * g.H * g.W * (int64_t)C * 2);
  a.wt_bytes = (uint32_t)(nw * 2);
  return stat_partials ? launch_igemm_w<0, true, 1, false, 0>(a, s) : launch_igemm_w<0, false, 1, false, 0>(a, s);
}

void conv_grouped_dgrad_mfma(const bf16_t* dy, const bf16_t* w, bf16_t* wd, bf16_t* dx, const ConvGeom& g, int groups,
                             bool accumulate, hipStream_t s) {
  const int C = g.Cin, cg = C / groups, SW = grouped_mfma_slice(C, groups);
  IgemmArgs a;
  fill_sliced(a, C, SW);
  a.stat_partials = nullptr;
  a.src = dy; a.dst = dx;
  a.Hs = g.Ho; a.Ws = g.Wo;
  a.src_bytes = (uint32_t)(g.M() * (int64_t)C * 2);
  a.Ho = g.H; a.Wo = g.W;
  if (g.stride == 1) {
    const int64_t nw = (int64_t)C * g.kh * g.kw * SW;
    hipLaunchKernelGGL(expand_sliced_weights_k<true>, dim3((unsigned)cdiv(nw, 256)), dim3(256), 0, s, w, wd, C, g.kh, g.kw, cg,
                       SW, g.kh, g.kw, 0, 0, 1);
    a.wt = wd;
    a.M = g.B * g.H * g.W; a.K = g.kh * g.kw * SW;
    a.Hd = g.H; a.Wd = g.W;
    a.kh = g.kh; a.kw = g.kw; a.stride = 1; a.pad = g.pad; a.pad_w = g.pad;
    a.accumulate = accumulate ? 1 : 0;
    a.wt_bytes = (uint32_t)(nw * 2);
    launch_igemm_w<1, false, 1, false, 0>(a, s);
    return;
  }
  // stride 2: one stride-1 problem per parity class of the input pixel, as in conv_dgrad_mfma
  bool covered_all = true;
  for (int ph = 0; ph < 2; ph++) {
    const int tmax = (ph + g.pad) >> 1, lo = ph + g.pad - g.kh + 1;
    if (tmax < (lo <= 0 ? -((-lo) >> 1) : (lo + 1) >> 1)) covered_all = false;
  }
  if (!accumulate && !covered_all) {
    const int64_t n16 = g.B * g.H * g.W * (int64_t)C / 8;
    hipLaunchKernelGGL(fill_zero16_k, dim3((unsigned)cdiv(n16, 256)), dim3(256), 0, s, reinterpret_cast<uint4*>(dx), n16);
    accumulate = true;
  }
  int64_t woff = 0;
  for (int ph = 0; ph < 2; ph++)
    for (int pw = 0; pw < 2; pw++) {
      const int loh = ph + g.pad - g.kh + 1, low = pw + g.pad - g.kw + 1;
      const int tminh = loh <= 0 ? -((-loh) >> 1) : (loh + 1) >> 1, tmaxh = (ph + g.pad) >> 1;
      const int tminw = low <= 0 ? -((-low) >> 1) : (low + 1) >> 1, tmaxw = (pw + g.pad) >> 1;
      const int th = tmaxh - tminh + 1, tw = tmaxw - tminw + 1;
      const int hd = (g.H - ph + 1) / 2, wdd = (g.W - pw + 1) / 2;
      if (th <= 0 || tw <= 0 || hd <= 0 || wdd <= 0) continue;
      bf16_t* wc = wd + woff;
      const int64_t wn = (int64_t)C * th * tw * SW;
      hipLaunchKernelGGL(expand_sliced_weights_k<true>, dim3((unsigned)cdiv(wn, 256)), dim3(256), 0, s, w, wc, C, g.kh, g.kw, cg,
                         SW, th, tw, ph + g.pad - 2 * tminh, pw + g.pad - 2 * tminw, -2);
      woff += (wn + 7) / 8 * 8;
      a.wt = wc;
      a.M = g.B * hd * wdd; a.K = th * tw * SW;
      a.Hd = hd; a.Wd = wdd;
      a.kh = th; a.kw = tw; a.stride = 1; a.pad = -tminh; a.pad_w = -tminw;
      a.omul = 2; a.ooff_h = ph; a.ooff_w = pw;
      a.accumulate = accumulate ? 1 : 0;
      a.wt_bytes = (uint32_t)(wn * 2);
      launch_igemm_w<0, false, 1, true, 0>(a, s);
    }
}

// ---- wgrad ------------------------------------------------------------------------------------------
// dw[n][k] = sum_m dy[m][n] * im2col(x)[m][k].  The contraction runs over pixels, which is the slow
// axis of both operands in memory.  Tiles are staged in LDS as they lie in memory ([pixel][channel],
// 16-byte vectors along the channels) and read back with the gfx950 LDS transpose load
// (ds_read_b64_tr_b16): in every group of 16 lanes, lane i receives element (i & 3) of the four
// 8-byte chunks addressed by lanes (i >> 2), 4 + (i >> 2), 8 + (i >> 2), 12 + (i >> 2).  Pointing
// chunk 4e+q at pixel e, channels 4q..4q+3 therefore hands lane i four consecutive pixels of channel
// i, which is the MFMA operand layout.  The pixel range is split over blockIdx.y; partial sums are
// written per split and added by a second kernel in a fixed order.
struct WgradArgs {
  const bf16_t* x;   // [B][H][W][Cin]
  const bf16_t* dy;  // [M][N]
  float* out;        // [splits][N][K]
  int64_t M, m_per_split;
  int N, K;
  int H, W, Cin, Ho, Wo, kh, kw, stride, pad;
  int ktiles, tiles;  // tiles along K; tiles of dw in all
  uint32_t x_bytes, dy_bytes;
  // Grouped convolutions (sliced launches): `slices` independent problems, slice s taking channels [s * N, (s + 1) * N) of
  // dy and [s * Cin, (s + 1) * Cin) of x, both row-major with `pitch` channels per pixel (N = Cin = the slice width);
  // out is [splits][slices][N][K].  An ordinary convolution: slices = 1, x_pitch = Cin, dy_pitch = N.
  int slices = 1, tiles_per_slice = 0, x_pitch = 0, dy_pitch = 0;
};

constexpr int WG_MS = 32;  // pixels per main-loop step

template <int BN, int BKK>
__global__ void __launch_bounds__(256) wgrad_kernel(WgradArgs a) {
  constexpr int PN = BN + 32, PK = BKK + 32;   // pitches (elements): rows 16 banks apart, conflict-free reads
  constexpr int NVR = BN / 8, KVR = BKK / 8;   // 16-byte vectors per tile row
  constexpr int DV = WG_MS * NVR / 256, XV = WG_MS * KVR / 256;  // vectors per thread per step
  constexpr int DROWS = 256 / NVR, XROWS = 256 / KVR;
  constexpr int WNT = BN / 2, WKT = BKK / 2;   // wave tile (2 x 2 waves)
  constexpr int TN = WNT / 32, TK = WKT / 32;
  __shared__ __attribute__((aligned(16))) bf16_t Dy[2][WG_MS][PN];
  __shared__ __attribute__((aligned(16))) bf16_t Xs[2][WG_MS][PK];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn0 = (wave & 1) * WNT, wk0 = (wave >> 1) * WKT;
  // One-dimensional grid of tiles x splits, renumbered per XCD: the tiles of one pixel range (they
  // read the same rows of dy, and the same rows of x up to the filter's reach) run side by side on
  // one XCD and share those rows in its L2 instead of each fetching them from memory.
  const unsigned wg = xcd_remap(blockIdx.x, gridDim.x);
  const unsigned split = wg / (unsigned)a.tiles, tile_all = wg - split * (unsigned)a.tiles;
  const unsigned sl = tile_all / (unsigned)a.tiles_per_slice, tile = tile_all - sl * (unsigned)a.tiles_per_slice;
  const int n0 = (int)(tile / (unsigned)a.ktiles) * BN, k0 = (int)(tile % (unsigned)a.ktiles) * BKK;
  const int dyc0 = (int)sl * a.N, xc0 = (int)sl * a.Cin;   // first channel of this slice in dy and in x
  // pixel and element indices fit 32 bits: every operand is smaller than 2 GiB (conv_mfma_supported)
  const int M = (int)a.M;
  const int mbeg = (int)split * (int)a.m_per_split;
  const int mend = mbeg + (int)a.m_per_split < M ? mbeg + (int)a.m_per_split : M;
  const __amdgpu_buffer_rsrc_t rx_src = make_rsrc(a.x, a.x_bytes);
  const __amdgpu_buffer_rsrc_t rdy = make_rsrc(a.dy, a.dy_bytes);

  // dy loader: fixed channel vector, DV rows; doff = byte offset of (row, channel vector) at step 0
  const int dnv = tid % NVR, drow = tid / NVR;
  const bool dnok = n0 + dnv * 8 < a.N;
  int dm[DV];
  uint32_t doff[DV];
#pragma unroll
  for (int j = 0; j < DV; j++) {
    dm[j] = mbeg + drow + DROWS * j;
    doff[j] = ((uint32_t)dm[j] * (uint32_t)a.dy_pitch + (uint32_t)(dyc0 + n0 + dnv * 8)) * 2u;
  }
  const uint32_t dstep = (uint32_t)WG_MS * (uint32_t)a.dy_pitch * 2u;
  // x loader: fixed (tap, channel) vector, XV rows, pixel coordinates advanced incrementally
  const int xkv = tid % KVR, xrow = tid / KVR;
  const int k = k0 + xkv * 8;
  const bool kok = k < a.K;
  const int tap = kok ? k / a.Cin : 0;
  const int kc = k - tap * a.Cin, kr = tap / a.kw, ks = tap - (tap / a.kw) * a.kw;
  int xm[XV], pb[XV], ph[XV], pw[XV];
#pragma unroll
  for (int j = 0; j < XV; j++) {
    const unsigned m = (unsigned)(mbeg + xrow + XROWS * j);
    const unsigned q = m / (unsigned)a.Wo;
    xm[j] = (int)m;
    pw[j] = (int)(m - q * (unsigned)a.Wo);
    pb[j] = (int)(q / (unsigned)a.Ho);
    ph[j] = (int)(q - (unsigned)pb[j] * (unsigned)a.Ho);
  }
  // one step moves every row WG_MS pixels on: whole images, then whole rows, then columns
  const int adv_b = WG_MS / (a.Ho * a.Wo), adv_r = WG_MS % (a.Ho * a.Wo);
  const int adv_h = adv_r / a.Wo, adv_w = adv_r % a.Wo;

  // Loads are unconditional (masked vectors read nothing) so that the compiler can count the loads in
  // flight, and the address update is straight-line code (selects, no loops); see igemm_kernel.
  uint4 rd[2][DV], rx[2][XV];
  auto gload = [&](uint4* rd, uint4* rx) {
#pragma unroll
    for (int j = 0; j < DV; j++) {
      rd[j] = buf_load16(rdy, (dnok && dm[j] < mend) ? doff[j] : 0xffffffffu);
      dm[j] += WG_MS;
      doff[j] += dstep;
    }
#pragma unroll
    for (int j = 0; j < XV; j++) {
      const int hi = ph[j] * a.stride - a.pad + kr, wi = pw[j] * a.stride - a.pad + ks;
      const bool ok = kok && xm[j] < mend && (unsigned)hi < (unsigned)a.H && (unsigned)wi < (unsigned)a.W;
      rx[j] = buf_load16(rx_src, ok ? (uint32_t)(((pb[j] * a.H + hi) * a.W + wi) * a.x_pitch + xc0 + kc) * 2u : 0xffffffffu);
      xm[j] += WG_MS;
      pw[j] += adv_w;
      const int cw = pw[j] >= a.Wo ? 1 : 0;
      pw[j] -= cw ? a.Wo : 0;
      ph[j] += adv_h + cw;
      const int ch = ph[j] >= a.Ho ? 1 : 0;
      ph[j] -= ch ? a.Ho : 0;
      pb[j] += adv_b + ch;
    }
  };
  auto lstore = [&](const uint4* rd, const uint4* rx, int buf) {
#pragma unroll
    for (int j = 0; j < DV; j++) *reinterpret_cast<uint4*>(&Dy[buf][drow + DROWS * j][dnv * 8]) = rd[j];
#pragma unroll
    for (int j = 0; j < XV; j++) *reinterpret_cast<uint4*>(&Xs[buf][xrow + XROWS * j][xkv * 8]) = rx[j];
  };

  f32x16_t acc[TN][TK];
#pragma unroll
  for (int i = 0; i < TN; i++)
#pragma unroll
    for (int j = 0; j < TK; j++)
#pragma unroll
      for (int v = 0; v < 16; v++) acc[i][j][v] = 0.f;

  // transpose-load addressing of this lane inside a 16-pixel x 32-channel fragment
  const int grp = lane >> 4, li = lane & 15;
  const int tr_m = 8 * (grp >> 1) + (li >> 2);      // pixel row (second load: +4)
  const int tr_c = 16 * (grp & 1) + 4 * (li & 3);   // first of the 4 channels this lane points at

  bf16x8_t df[2][2][TN], xf[2][2][TK];  // [fragment set][16-pixel half][tile]
  auto read_frags = [&](bf16x8_t (&df)[2][TN], bf16x8_t (&xf)[2][TK], int buf) {
#pragma unroll
    for (int h = 0; h < 2; h++) {
#pragma unroll
      for (int i = 0; i < TN; i++) {
        const bf16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (CD_LDS bf16x4_t*)(&Dy[buf][h * 16 + tr_m][wn0 + i * 32 + tr_c]));
        const bf16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (CD_LDS bf16x4_t*)(&Dy[buf][h * 16 + tr_m + 4][wn0 + i * 32 + tr_c]));
        df[h][i] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
#pragma unroll
      for (int j = 0; j < TK; j++) {
        const bf16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (CD_LDS bf16x4_t*)(&Xs[buf][h * 16 + tr_m][wk0 + j * 32 + tr_c]));
        const bf16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            (CD_LDS bf16x4_t*)(&Xs[buf][h * 16 + tr_m + 4][wk0 + j * 32 + tr_c]));
        xf[h][j] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      }
    }
  };
  auto mfma_step = [&](const bf16x8_t (&df)[2][TN], const bf16x8_t (&xf)[2][TK]) {
#pragma unroll
    for (int h = 0; h < 2; h++)
#pragma unroll
      for (int i = 0; i < TN; i++)
#pragma unroll
        for (int j = 0; j < TK; j++)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(df[h][i], xf[h][j], acc[i][j], 0, 0, 0);
  };

  // same software pipeline as igemm_kernel: store tile st+1, load tile st+3, MFMAs of tile st, barrier,
  // fragments of tile st+1
  auto interleave = [&]() {
    constexpr int NMFMA = 2 * TN * TK, NREAD = 4 * (TN + TK), NWRITE = DV + XV;
#pragma unroll
    for (int i = 0; i < NMFMA; i++) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                  // MFMA
      __builtin_amdgcn_sched_group_barrier(0x100, (NREAD + NMFMA - 1) / NMFMA, 0);        // DS read
      __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);                                  // VALU
      if (i < NWRITE) {
        __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                                // DS write
        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                                // VMEM read
      }
    }
  };
  const int steps = (mend - mbeg + WG_MS - 1) / WG_MS;
  gload(rd[0], rx[0]);
  gload(rd[1], rx[1]);
  lstore(rd[0], rx[0], 0);
  gload(rd[0], rx[0]);
  __syncthreads();
  read_frags(df[0], xf[0], 0);
  for (int st = 0; st < steps; st += 2) {
    lstore(rd[1], rx[1], 1);
    gload(rd[1], rx[1]);
    mfma_step(df[0], xf[0]);
    interleave();
    __syncthreads();
    read_frags(df[1], xf[1], 1);
    lstore(rd[0], rx[0], 0);
    gload(rd[0], rx[0]);
    mfma_step(df[1], xf[1]);
    interleave();
    __syncthreads();
    read_frags(df[0], xf[0], 0);
  }

  float* out = a.out + ((int64_t)split * a.slices + sl) * a.N * a.K;   // N*K*4 bytes < 2^33: 32-bit element offsets inside
#pragma unroll
  for (int i = 0; i < TN; i++)
#pragma unroll
    for (int j = 0; j < TK; j++) {
      const int kk = k0 + wk0 + j * 32 + (lane & 31);
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int n = n0 + wn0 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        if (n < a.N && kk < a.K) out[(uint32_t)n * (uint32_t)a.K + (uint32_t)kk] = acc[i][j][v];
      }
    }
}

// 64 outputs x 4 split lanes per block; every lane adds every 4th split, fixed-order combine in LDS
__global__ void __launch_bounds__(256) wgrad_reduce_kernel(const float* __restrict__ part, float* __restrict__ out,
                                                           int64_t n, int splits) {
  __shared__ float sm[4][64];
  const int ol = threadIdx.x & 63, lane = threadIdx.x >> 6;
  const int64_t i = (int64_t)blockIdx.x * 64 + ol;
  float s = 0.f;
  if (i < n) {
#pragma unroll 8
    for (int j = lane; j < splits; j += 4) s += part[(int64_t)j * n + i];
  }
  sm[lane][ol] = s;
  __syncthreads();
  if (lane == 0 && i < n) out[i] = (sm[0][ol] + sm[1][ol]) + (sm[2][ol] + sm[3][ol]);
}

// slices > 1: a grouped convolution cut into `slices` slices of g.Cin = g.Cout = SW channels; x and dy are the whole
// row-major tensors with `pitch` channels per pixel and dw receives the dense per-slice gradients [slices][SW][K].
static void wgrad_launch(const bf16_t* x, const bf16_t* dy, float* dw, const ConvGeom& g, int slices, int pitch, float* partials,
                         size_t partials_bytes, hipStream_t s) {
  WgradArgs a;
  a.x = x; a.dy = dy;
  a.M = g.M(); a.N = g.Cout; a.K = g.K();
  a.H = g.H; a.W = g.W; a.Cin = g.Cin; a.Ho = g.Ho; a.Wo = g.Wo;
  a.kh = g.kh; a.kw = g.kw; a.stride = g.stride; a.pad = g.pad;
  a.slices = slices;
  a.x_pitch = slices > 1 ? pitch : g.Cin;
  a.dy_pitch = slices > 1 ? pitch : g.Cout;
  a.x_bytes = (uint32_t)(g.B * g.H * g.W * (int64_t)a.x_pitch * 2);
  a.dy_bytes = (uint32_t)(g.M() * (int64_t)a.dy_pitch * 2);
  const int bn = a.N > 64 ? 128 : 64, bk = a.K > 64 ? 128 : 64;
  const int ntiles = (int)cdiv(a.N, bn);
  a.ktiles = (int)cdiv(a.K, bk);
  a.tiles_per_slice = ntiles * a.ktiles;
  const int64_t tiles = (int64_t)a.tiles_per_slice * slices;
  const int64_t nk = (int64_t)a.N * a.K * slices;
  // Workgroups to aim for (measured on the layer shapes of ResNet-50 at batch 256).  Every split writes
  // an fp32 copy of dw, so 1x1 filters with small N*K/(N+K) (few flops per byte of dy and x: the launch
  // is bound by memory traffic whatever the split) run one long workgroup per compute unit; the other
  // 1x1 launches take two, gathers over several taps four.
  int64_t target = 1024;
  if (a.kh * a.kw == 1) target = (double)a.N * a.K / ((double)a.N + a.K) < 150.0 ? 256 : 512;
  if (g_tune_co > 0) target = g_tune_co;
  int64_t splits = cdiv(target, tiles);
  const int64_t max_by_m = cdiv(a.M, 4 * WG_MS);
  if (splits > max_by_m) splits = max_by_m;
  const int64_t max_by_mem = (int64_t)(partials_bytes / (nk * sizeof(float)));
  if (splits > max_by_mem) splits = max_by_mem;
  if (splits < 1) splits = 1;
  a.m_per_split = cdiv(cdiv(a.M, splits), WG_MS) * WG_MS;
  splits = cdiv(a.M, a.m_per_split);
  a.out = splits == 1 ? dw : partials;
  a.tiles = (int)tiles;
  dim3 grid((unsigned)(tiles * splits));
  if (bn == 128 && bk == 128) hipLaunchKernelGGL((wgrad_kernel<128, 128>), grid, dim3(256), 0, s, a);
  else if (bn == 128) hipLaunchKernelGGL((wgrad_kernel<128, 64>), grid, dim3(256), 0, s, a);
  else if (bk == 128) hipLaunchKernelGGL((wgrad_kernel<64, 128>), grid, dim3(256), 0, s, a);
  else hipLaunchKernelGGL((wgrad_kernel<64, 64>), grid, dim3(256), 0, s, a);
  if (splits > 1)
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)cdiv(nk, 64)), dim3(256), 0, s, partials, dw, nk,
                       (int)splits);
}

void conv_wgrad_mfma(const bf16_t* x, const bf16_t* dy, float* dw, const ConvGeom& g, float* partials,
                     size_t partials_bytes, hipStream_t s) {
  wgrad_launch(x, dy, dw, g, 1, 0, partials, partials_bytes, s);
}

// dw [C][taps][cg] fp32 of a grouped convolution: dense per-slice gradients dwd [C / SW][SW][taps][SW] (scratch) by the
// sliced launch, then the diagonal blocks.
__global__ void __launch_bounds__(256) extract_sliced_dw_k(const float* __restrict__ dwd, float* __restrict__ dw, int C,
                                                           int taps, int cg, int SW) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)C * taps * cg) return;
  const int j = (int)(idx % cg);
  const int t = (int)((idx / cg) % taps);
  const int o = (int)(idx / ((int64_t)cg * taps));
  dw[idx] = dwd[((int64_t)o * taps + t) * SW + (o % SW) / cg * cg + j];
}

void conv_grouped_wgrad_mfma(const bf16_t* x, const bf16_t* dy, float* dwd, float* dw, const ConvGeom& g, int groups,
                             float* partials, size_t partials_bytes, hipStream_t s) {
  const int C = g.Cin, cg = C / groups, SW = grouped_mfma_slice(C, groups), taps = g.kh * g.kw;
  ConvGeom gs = g;
  gs.Cin = gs.Cout = SW;
  wgrad_launch(x, dy, dwd, gs, C / SW, C, partials, partials_bytes, s);
  const int64_t n = (int64_t)C * taps * cg;
  hipLaunchKernelGGL(extract_sliced_dw_k, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s, dwd, dw, C, taps, cg, SW);
}

// eight elements per thread (two 16-byte loads, one 16-byte store); the ragged tail element by element
__global__ void __launch_bounds__(256) cast_f32_bf16_k(const float* __restrict__ in, bf16_t* __restrict__ out, int64_t n) {
  const int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i + 8 <= n) {
    const float4 a = *reinterpret_cast<const float4*>(in + i), b = *reinterpret_cast<const float4*>(in + i + 4);
    *reinterpret_cast<uint4*>(out + i) =
        make_uint4(pack_bf16x2(a.x, a.y), pack_bf16x2(a.z, a.w), pack_bf16x2(b.x, b.y), pack_bf16x2(b.z, b.w));
  } else {
    for (int64_t j = i; j < n; j++) out[j] = f32_to_bf16(in[j]);
  }
}
void cast_f32_bf16(const float* in, bf16_t* out, int64_t n, hipStream_t s) {   // in, out 16-byte aligned
  hipLaunchKernelGGL(cast_f32_bf16_k, dim3((unsigned)cdiv(cdiv(n, 8), 256)), dim3(256), 0, s, in, out, n);
}

// ---- layout helpers ---------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) pad_c3_to_c8_k(const bf16_t* __restrict__ in, bf16_t* __restrict__ out,
                                                      int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  const uint32_t a = in[3 * i], b = in[3 * i + 1], c = in[3 * i + 2];
  reinterpret_cast<uint4*>(out)[i] = make_uint4(a | (b << 16), c, 0u, 0u);
}
void pad_c3_to_c8(const bf16_t* in, bf16_t* out, int64_t n, hipStream_t s) {
  hipLaunchKernelGGL(pad_c3_to_c8_k, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s, in, out, n);
}
// ---- space-to-depth form of a stride-2 convolution on 3-channel images ------------------------------
// x[b][2I+p][2J+q][c] -> xs[b][I][J][(2p+q)*3 + c] (16 channels, the last four zero): a k x k stride-2
// filter with padding pad becomes a ks x ks stride-1 filter on xs with padding P = ceil(pad / 2),
// ks = ceil((k + 2P - pad) / 2), whose tap (R, S), channel (2p+q)*3 + c is the original tap
// r = 2R + p - (2P - pad), s = 2S + q - (2P - pad) (zero where that falls outside the filter).  The
// contraction shrinks from k*k*8 (channels padded to a 16-byte vector) to ks*ks*16.
__global__ void __launch_bounds__(256) s2d_pack_x_k(const bf16_t* __restrict__ x, bf16_t* __restrict__ xs, int64_t n,
                                                    int Hs, int Ws) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;  // (b, I, J)
  if (i >= n) return;
  const int J = (int)(i % Ws);
  const int64_t q = i / Ws;
  const int I = (int)(q % Hs);
  const int64_t b = q / Hs;
  const int W = 2 * Ws;
  const bf16_t* r0 = x + ((b * 2 * Hs + 2 * I) * W + 2 * J) * 3;  // six contiguous elements per image row
  const bf16_t* r1 = r0 + (int64_t)W * 3;
  uint32_t u[8];
  u[0] = r0[0] | ((uint32_t)r0[1] << 16); u[1] = r0[2] | ((uint32_t)r0[3] << 16); u[2] = r0[4] | ((uint32_t)r0[5] << 16);
  u[3] = r1[0] | ((uint32_t)r1[1] << 16); u[4] = r1[2] | ((uint32_t)r1[3] << 16); u[5] = r1[4] | ((uint32_t)r1[5] << 16);
  u[6] = 0; u[7] = 0;
  uint4* o = reinterpret_cast<uint4*>(xs + i * 16);
  o[0] = make_uint4(u[0], u[1], u[2], u[3]);
  o[1] = make_uint4(u[4], u[5], u[6], u[7]);
}
void s2d_pack_x(const bf16_t* x, bf16_t* xs, int64_t B, int H, int W, hipStream_t s) {
  const int64_t n = B * (H / 2) * (W / 2);
  hipLaunchKernelGGL(s2d_pack_x_k, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s, x, xs, n, H / 2, W / 2);
}
// w[n][k][k][3] -> ws[n][ks][ks][16]
__global__ void __launch_bounds__(256) s2d_pack_w_k(const bf16_t* __restrict__ w, bf16_t* __restrict__ ws, int cout,
                                                    int k, int ks, int shift) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= cout * ks * ks * 16) return;
  const int ch = i & 15, S = (i >> 4) % ks, R = (i >> 4) / ks % ks, n = (i >> 4) / (ks * ks);
  bf16_t v = 0;
  if (ch < 12) {
    const int pq = ch / 3, c = ch - pq * 3;
    const int r = 2 * R + (pq >> 1) - shift, t = 2 * S + (pq & 1) - shift;
    if (r >= 0 && r < k && t >= 0 && t < k) v = w[((n * k + r) * k + t) * 3 + c];
  }
  ws[i] = v;
}
void s2d_pack_w(const bf16_t* w, bf16_t* ws, int cout, int k, int ks, int shift, hipStream_t s) {
  hipLaunchKernelGGL(s2d_pack_w_k, dim3((unsigned)cdiv(cout * ks * ks * 16, 256)), dim3(256), 0, s, w, ws, cout, k, ks,
                     shift);
}
// fp32 dws[n][ks][ks][16] -> dw[n][k][k][3]
__global__ void __launch_bounds__(256) s2d_unpack_dw_k(const float* __restrict__ dws, float* __restrict__ dw, int cout,
                                                       int k, int ks, int shift) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= cout * k * k * 3) return;
  const int c = i % 3, t = i / 3 % k, r = i / 3 / k % k, n = i / 3 / (k * k);
  const int rr = r + shift, tt = t + shift;
  dw[i] = dws[((n * ks + (rr >> 1)) * ks + (tt >> 1)) * 16 + ((rr & 1) * 2 + (tt & 1)) * 3 + c];
}
void s2d_unpack_dw(const float* dws, float* dw, int cout, int k, int ks, int shift, hipStream_t s) {
  hipLaunchKernelGGL(s2d_unpack_dw_k, dim3((unsigned)cdiv(cout * k * k * 3, 256)), dim3(256), 0, s, dws, dw, cout, k, ks,
                     shift);
}

__global__ void __launch_bounds__(256) unpad_c8_to_c3_k(const float* __restrict__ in, float* __restrict__ out,
                                                        int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= 3 * n) return;
  out[i] = in[(i / 3) * 8 + i % 3];
}
void unpad_c8_to_c3(const float* in, float* out, int64_t n, hipStream_t s) {
  hipLaunchKernelGGL(unpad_c8_to_c3_k, dim3((unsigned)cdiv(3 * n, 256)), dim3(256), 0, s, in, out, n);
}
__global__ void __launch_bounds__(256) transpose_weight_k(const bf16_t* __restrict__ w, bf16_t* __restrict__ wt,
                                                          int cout, int taps, int cin) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)cout * taps * cin) return;
  const int n = i % cout;
  const int64_t q = i / cout;
  const int tap = q % taps;
  const int c = q / taps;
  wt[i] = w[((int64_t)n * taps + tap) * cin + c];
}
void transpose_weight(const bf16_t* w, bf16_t* wt, int cout, int taps, int cin, hipStream_t s) {
  const int64_t n = (int64_t)cout * taps * cin;
  hipLaunchKernelGGL(transpose_weight_k, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, s, w, wt, cout, taps, cin);
}

}  // namespace cd
