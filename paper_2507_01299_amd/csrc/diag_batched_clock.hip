// Diagnostic program (not part of liblarosa): the batched path's two kernels -- the matrix-core projection over all
// weight rows and the per-token Top-K kernel -- on the shapes of a LLaMA3-8B-shaped decoder layer, bf16, built with the
// phase clocks compiled in.  For every shape it prints the event-timed launch time and where inside the launch the
// time goes.  Weights are hashed pseudo-random and rotated over enough copies to defeat the caches; the vectors the
// Top-K kernel selects from are sums of uniform variates; the only check is that no token keeps more than K values
// (parity is the tests' business).
//
// Build and run:  python -m paper_2507_01299_amd.build --diag  &&  paper_2507_01299_amd/_build/diag_batched_clock
// Options: --batch N (tokens, default 16), --g N (workgroups a projection launch aims for), --reps N, --only NAME.
#define LAROSA_PHASE_CLOCK 1
#include "batched.hip"
#include "topk.hip"
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)
using namespace larosa;
namespace larosa { Tuning& tuning() { static Tuning t; return t; } }

static inline uint32_t hashu(uint32_t x) { x ^= x >> 15; x *= 2246822519u; x ^= x >> 13; x *= 3266489917u; x ^= x >> 16; return x; }
static uint16_t f2bf(float f) { uint32_t u; memcpy(&u, &f, 4); u += 0x7FFF + ((u >> 16) & 1); return (uint16_t)(u >> 16); }
static float bellish(uint32_t i) { float s = 0; for (int k = 0; k < 6; ++k) s += (hashu(i * 6 + k) & 0xFFFF) / 65536.0f - 0.5f; return s * 1.4f; }
__global__ void fill_bf16(uint16_t* w, size_t n, unsigned seed) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, st = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += st) {
    uint32_t x = (uint32_t)i * 2654435761u + seed; x ^= x >> 15; x *= 2246822519u; x ^= x >> 13; x *= 3266489917u; x ^= x >> 16;
    const uint32_t u = __float_as_uint(((x & 0xFFFF) / 65536.0f - 0.5f) * 0.07f);
    w[i] = (uint16_t)((u + 0x7FFF + ((u >> 16) & 1)) >> 16);
  }
}

int main(int argc, char** argv) {
  int G = 0, reps = 30, B = 16; const char* only = nullptr;
  for (int i = 1; i < argc; ++i) {
    if (!strcmp(argv[i], "--g") && i + 1 < argc) G = atoi(argv[++i]);
    else if (!strcmp(argv[i], "--reps") && i + 1 < argc) reps = atoi(argv[++i]);
    else if (!strcmp(argv[i], "--only") && i + 1 < argc) only = argv[++i];
    else if (!strcmp(argv[i], "--batch") && i + 1 < argc) B = atoi(argv[++i]);
  }
  if (B < 2 || B > 32 || reps < 1 || reps > 1000 || G < 0 || G > 2048) { printf("--batch 2..32, --reps 1..1000, --g 0..2048\n"); return 1; }
  const int maxwg = 4096;
  unsigned long long* dbg; CK(hipMalloc(&dbg, (size_t)maxwg * kPhaseSlots * 8));
  CK(hipMemcpyToSymbol(HIP_SYMBOL(larosa_phase_clock), &dbg, sizeof(dbg)));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));

  // ---- batched projections ------------------------------------------------------------------------------------
  struct Shape { const char* n; int d_in, d_out; } shapes[] = {{"o", 4096, 4096}, {"qkv", 4096, 6144}, {"down", 14336, 4096}, {"gu", 4096, 28672}};
  unsigned* ctr; CK(hipMalloc(&ctr, 1 << 20)); CK(hipMemset(ctr, 0, 1 << 20));
  float* partial; CK(hipMalloc(&partial, 256u << 20));
  for (auto& sh : shapes) {
    if (only && strcmp(only, sh.n)) continue;
    const size_t wn = (size_t)sh.d_in * sh.d_out, wb = wn * 2;
    const int nset = (int)std::min<size_t>(24, std::max<size_t>(3, (800u << 20) / wb + 1));
    std::vector<uint16_t*> W(nset);
    for (int i = 0; i < nset; ++i) { CK(hipMalloc(&W[i], wb)); hipLaunchKernelGGL(fill_bf16, dim3(4096), dim3(256), 0, 0, W[i], wn, 10u + i); }
    uint16_t *C, *y; CK(hipMalloc(&C, (size_t)32 * sh.d_in * 2)); CK(hipMalloc(&y, (size_t)32 * sh.d_out * 2));
    hipLaunchKernelGGL(fill_bf16, dim3(256), dim3(256), 0, 0, C, (size_t)32 * sh.d_in, 999u);
    CK(hipDeviceSynchronize());
    const GemvPlan p = plan_batched(sh.d_in, sh.d_out, true, G);
    BatchArgs a{}; a.C = C; a.y = y; a.d_in = sh.d_in; a.d_out = sh.d_out; a.B = B;
    a.chunk = p.chunk; a.G = p.G; a.nstrips = p.nstrips; a.wps = p.wps; a.counters = ctr; a.partial = partial;
    const size_t need = (size_t)32 * p.partial_floats * sizeof(float);
    if (p.G > maxwg || need > (256u << 20) || (size_t)p.nstrips * kCounterStride * 4 > (1u << 20)) { printf("%s: launch plan too large for this program\n", sh.n); return 1; }
    double ev = 0, rows_avg = 0, rows_max = 0, store = 0, arrive = 0, fin = 0, end = 0, start = 0;
    for (int r = 0; r < reps + 4; ++r) {
      a.W = W[r % nset];
      CK(hipMemset(dbg, 0, (size_t)maxwg * kPhaseSlots * 8));
      CK(hipEventRecord(e0, 0));
      CK(launch_batched(a, true, 0));
      CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1));
      float ms; CK(hipEventElapsedTime(&ms, e0, e1));
      if (r < 4) continue;
      ev += ms * 1e3;
      std::vector<unsigned long long> h((size_t)p.G * kPhaseSlots);
      CK(hipMemcpy(h.data(), dbg, h.size() * 8, hipMemcpyDeviceToHost));
      unsigned long long t0 = ~0ull; for (int g = 0; g < p.G; ++g) t0 = std::min(t0, h[(size_t)g * kPhaseSlots]);
      double sa = 0, sm = 0, st = 0, sc = 0, sf = 0, se = 0, ss = 0; int nf = 0;
      for (int g = 0; g < p.G; ++g) {
        const unsigned long long* q = &h[(size_t)g * kPhaseSlots];
        ss = std::max(ss, (q[0] - t0) * 0.01);
        sa += (q[1] - t0) * 0.01; sm = std::max(sm, (q[1] - t0) * 0.01);
        if (q[2]) { st += (q[2] - q[1]) * 0.01; sc += (q[3] - q[2]) * 0.01; nf++; }
        se = std::max(se, (q[5] - t0) * 0.01);
        if (q[3]) sf = std::max(sf, (q[5] - q[3]) * 0.01);
      }
      start += ss; rows_avg += sa / p.G; rows_max += sm; if (nf) { store += st / nf; arrive += sc / nf; } fin += sf; end += se;
    }
    printf("%-5s B=%d G=%d chunk=%d strips=%d  event %6.2f us (%.2f TB/s) | last start %.2f, rows done avg %.2f max %.2f, sum+store %.2f, arrive %.2f, finisher tail max %.2f, last end %.2f\n",
           sh.n, B, p.G, p.chunk, p.nstrips, ev / reps, wb / (ev / reps) * 1e-6, start / reps, rows_avg / reps, rows_max / reps,
           store / reps, arrive / reps, fin / reps, end / reps);
    for (int i = 0; i < nset; ++i) CK(hipFree(W[i]));
    CK(hipFree(C)); CK(hipFree(y));
  }

  // ---- per-token Top-K -------------------------------------------------------------------------------------------
  struct Case { const char* n; int d, K, mode; bool want_idx; } cases[] = {
    {"topk plain d=4096", 4096, 2458, kSrcPlain, false}, {"topk plain d=4096 +idx", 4096, 2458, kSrcPlain, true},
    {"topk norm d=4096", 4096, 2458, kSrcNorm, false},
    {"topk silu d=14336", 14336, 8602, kSrcSilu, false}, {"topk silu d=14336 +idx", 14336, 8602, kSrcSilu, true},
    {"topk plain d=14336", 14336, 8602, kSrcPlain, false}};
  for (auto& c : cases) {
    if (only && strncmp(only, "topk", 4)) continue;
    const size_t n = (size_t)B * c.d * (c.mode == kSrcSilu ? 2 : 1);
    std::vector<uint16_t> hv(n);
    for (size_t i = 0; i < n; ++i) hv[i] = f2bf(bellish((uint32_t)i + 77u * c.d));
    uint16_t *src, *hout, *masked, *scale; int32_t* idx;
    CK(hipMalloc(&src, n * 2)); CK(hipMalloc(&hout, (size_t)B * c.d * 2)); CK(hipMalloc(&masked, (size_t)B * c.d * 2));
    CK(hipMalloc(&scale, c.d * 2)); CK(hipMalloc(&idx, (size_t)B * c.K * 4));
    CK(hipMemcpy(src, hv.data(), n * 2, hipMemcpyHostToDevice));
    std::vector<uint16_t> ones(c.d, f2bf(1.0f)); CK(hipMemcpy(scale, ones.data(), c.d * 2, hipMemcpyHostToDevice));
    TopkSource sc{}; sc.mode = c.mode; sc.src = src; sc.h_out = hout; sc.norm_scale = scale; sc.norm_eps = 1e-5f;
    double ph[5] = {0, 0, 0, 0, 0}, ev = 0;
    for (int r = 0; r < reps + 4; ++r) {
      CK(hipMemset(dbg, 0, 64 * kPhaseSlots * 8));
      CK(hipEventRecord(e0, 0));
      CK(launch_topk_from(sc, B, c.d, c.K, c.want_idx ? idx : nullptr, masked, true, 0));
      CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1));
      float ms; CK(hipEventElapsedTime(&ms, e0, e1));
      if (r < 4) continue;
      ev += ms * 1e3;
      std::vector<unsigned long long> h((size_t)B * kPhaseSlots);
      CK(hipMemcpy(h.data(), dbg, h.size() * 8, hipMemcpyDeviceToHost));
      unsigned long long t0 = ~0ull; for (int b = 0; b < B; ++b) t0 = std::min(t0, h[b * kPhaseSlots]);
      for (int k = 0; k < 5; ++k) { unsigned long long m = 0; for (int b = 0; b < B; ++b) m = std::max(m, h[b * kPhaseSlots + k]); ph[k] += (m - t0) * 0.01; }
    }
    printf("%-24s event %6.2f us | phase ends of the last workgroup (us from the first start): start %5.2f vector %5.2f select %5.2f emit %5.2f stores %5.2f\n",
           c.n, ev / reps, ph[0] / reps, ph[1] / reps, ph[2] / reps, ph[3] / reps, ph[4] / reps);
    std::vector<uint16_t> mk((size_t)B * c.d); CK(hipMemcpy(mk.data(), masked, mk.size() * 2, hipMemcpyDeviceToHost));
    int bad = 0;
    for (int b = 0; b < B; ++b) { int nz = 0; for (int j = 0; j < c.d; ++j) nz += (mk[(size_t)b * c.d + j] & 0x7FFF) != 0; if (nz > c.K) bad++; }
    if (bad) printf("  !! %d tokens keep more than K values\n", bad);
    CK(hipFree(src)); CK(hipFree(hout)); CK(hipFree(masked)); CK(hipFree(scale)); CK(hipFree(idx));
  }
  return 0;
}
