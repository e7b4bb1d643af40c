// Per-layer timing of the bf16 MFMA convolution kernels (forward, data gradient, weight gradient) on the layer shapes
// of ResNet-50 at a given batch size, each against the roofline of its own shape (max of flops / 2.5 PFLOP/s and
// bytes / 8 TB/s, every operand once).  A development aid: links libcodistill.so and calls the kernel launchers
// directly (not the C ABI).  Build and run:
//   python -m paper_2010_02838_amd.build --layer-bench && paper_2010_02838_amd/conv_layer_bench [batch [layer-name-filter
//   [tile [wgrad-workgroups [1 = with the BatchNorm column sums in the forward epilogue]]]]]
#include "kernels.h"
#include <cstdio>
#include <cstring>
#include <algorithm>
#include <cstdlib>
#include <vector>
#include <string>
using namespace cd;
namespace cd { extern int g_tune_tile, g_tune_co; }
struct L { const char* name; int count; int H, Cin, Cout, k, stride, pad; bool dgrad; };
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)
int main(int argc, char** argv) {
  int B = argc > 1 ? atoi(argv[1]) : 256;
  const char* only = argc > 2 && argv[2][0] ? argv[2] : nullptr;
  if (argc > 3) g_tune_tile = atoi(argv[3]);
  if (argc > 4) g_tune_co = atoi(argv[4]);
  const bool with_stats = argc > 5 && atoi(argv[5]);
  printf("tile %d co %d stats %d\n", g_tune_tile, g_tune_co, (int)with_stats);
  std::vector<L> layers = {
    {"stem7x7s2", 1, 224, 8, 64, 7, 2, 3, false},
    {"s1.c1 64>64 1x1", 1, 56, 64, 64, 1, 1, 0, true}, {"s1.c1 256>64 1x1", 2, 56, 256, 64, 1, 1, 0, true},
    {"s1.c2 3x3 64", 3, 56, 64, 64, 3, 1, 1, true}, {"s1.c3 64>256 1x1", 4, 56, 64, 256, 1, 1, 0, true},
    {"s2.c1 256>128", 1, 56, 256, 128, 1, 1, 0, true}, {"s2.c2 3x3s2 128", 1, 56, 128, 128, 3, 2, 1, true},
    {"s2.down 256>512 s2", 1, 56, 256, 512, 1, 2, 0, true}, {"s2.c3 128>512", 4, 28, 128, 512, 1, 1, 0, true},
    {"s2.c1 512>128", 3, 28, 512, 128, 1, 1, 0, true}, {"s2.c2 3x3 128", 3, 28, 128, 128, 3, 1, 1, true},
    {"s3.c1 512>256", 1, 28, 512, 256, 1, 1, 0, true}, {"s3.c2 3x3s2 256", 1, 28, 256, 256, 3, 2, 1, true},
    {"s3.down 512>1024 s2", 1, 28, 512, 1024, 1, 2, 0, true}, {"s3.c3 256>1024", 6, 14, 256, 1024, 1, 1, 0, true},
    {"s3.c1 1024>256", 5, 14, 1024, 256, 1, 1, 0, true}, {"s3.c2 3x3 256", 5, 14, 256, 256, 3, 1, 1, true},
    {"s4.c1 1024>512", 1, 14, 1024, 512, 1, 1, 0, true}, {"s4.c2 3x3s2 512", 1, 14, 512, 512, 3, 2, 1, true},
    {"s4.down 1024>2048 s2", 1, 14, 1024, 2048, 1, 2, 0, true}, {"s4.c3 512>2048", 3, 7, 512, 2048, 1, 1, 0, true},
    {"s4.c1 2048>512", 2, 7, 2048, 512, 1, 1, 0, true}, {"s4.c2 3x3 512", 2, 7, 512, 512, 3, 1, 1, true},
  };
  size_t maxact = (size_t)B * 112 * 112 * 64 * 2 + (size_t)B * 224 * 224 * 8 * 2;
  bf16_t *x, *y, *w, *wt; float *dw, *part;
  CK(hipMalloc(&x, maxact)); CK(hipMalloc(&y, maxact)); CK(hipMalloc(&w, 64 << 20)); CK(hipMalloc(&wt, 64 << 20));
  CK(hipMalloc(&dw, 64 << 20)); CK(hipMalloc(&part, kPartialsBytes));
  CK(hipMemset(x, 0x3c, maxact)); CK(hipMemset(y, 0x3c, maxact)); CK(hipMemset(w, 0x3c, 64 << 20)); CK(hipMemset(wt, 0x3c, 64 << 20));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  double tot[3] = {0, 0, 0}, ideal[3] = {0, 0, 0};
  printf("%-22s %3s | %8s %6s %6s | %8s %6s | %8s %6s | roof_us\n", "layer", "cnt", "fprop_us", "TF/s", "%roof", "dgrad_us", "%roof", "wgrad_us", "%roof");
  for (auto& l : layers) {
    if (only && !strstr(l.name, only)) continue;
    ConvGeom g; g.B = B; g.H = g.W = l.H; g.Cin = l.Cin; g.Cout = l.Cout; g.kh = g.kw = l.k; g.stride = l.stride; g.pad = l.pad;
    g.Ho = g.Wo = (l.H + 2 * l.pad - l.k) / l.stride + 1;
    double flops = 2.0 * g.M() * g.Cout * g.K();
    double bytes = 2.0 * ((double)B * g.H * g.W * g.Cin + (double)g.M() * g.Cout + (double)g.Cout * g.K());
    double roof = std::max(flops / 2.5e15, bytes / 8e12) * 1e6;
    float ms[3] = {0, 0, 0};
    for (int mode = 0; mode < 3; mode++) {
      if (mode == 1 && !l.dgrad) continue;
      const int reps = 5;
      for (int it = 0; it < reps + 2; it++) {
        if (it == 2) CK(hipEventRecord(e0, 0));
        if (mode == 0) conv_fprop_mfma(x, w, nullptr, false, y, g, with_stats ? part : nullptr, 0);
        else if (mode == 1) conv_dgrad_mfma(y, w, wt, x, g, false, 0);
        else conv_wgrad_mfma(x, y, dw, g, part, kPartialsBytes, 0);
      }
      CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1)); CK(hipGetLastError());
      CK(hipEventElapsedTime(&ms[mode], e0, e1)); ms[mode] /= reps;
      tot[mode] += ms[mode] * l.count * (mode == 0 ? 2 : 1);   // two forwards per step
      ideal[mode] += roof * 1e-3 * l.count * (mode == 0 ? 2 : 1);
    }
    printf("%-22s %3d | %8.1f %6.0f %5.0f%% | %8.1f %5.0f%% | %8.1f %5.0f%% | %7.1f\n", l.name, l.count, ms[0] * 1e3,
           flops / (ms[0] * 1e-3) / 1e12, 100 * roof / (ms[0] * 1e3), ms[1] * 1e3, ms[1] > 0 ? 100 * roof / (ms[1] * 1e3) : 0,
           ms[2] * 1e3, 100 * roof / (ms[2] * 1e3), roof);
  }
  printf("per step (2 fwd + 1 bwd): fprop %.2f ms (roof %.2f)  dgrad %.2f ms (roof %.2f)  wgrad %.2f ms (roof %.2f)  total %.2f ms (roof %.2f)\n",
         tot[0], ideal[0], tot[1], ideal[1], tot[2], ideal[2], tot[0] + tot[1] + tot[2], ideal[0] + ideal[1] + ideal[2]);
  return 0;
}
