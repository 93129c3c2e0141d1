// Diagnostic program (not part of liblarosa): the library's projection kernel with the Top-K prologue on
// the four projection shapes of a LLaMA2-7B-shaped decoder layer (q|k|v and gate|up also with the shortcut
// adapter as a side job of the same launch), built with the phase clocks compiled in.  For every launch
// shape it prints the event-timed launch time, the span from the first workgroup's start to the last
// workgroup's end, where in the kernel the time goes (vector ready / select done / row list ready / rows
// streamed / partial handed over / finished), and checks the Top-K indices and 48 output columns against a
// plain host computation.  Inputs are hashed pseudo-random weights and a heavy-tailed activation vector.
//
// Build and run:  python -m paper_2507_01299_amd.build --diag  &&  paper_2507_01299_amd/_build/diag_phase_clock
// Options: --gmain N / --gside N (workgroups of the projection / of the adapter), --only NAME, --reps N,
//          --hint (the down projection takes its threshold from host-built key histograms; gate|up builds
//          them and they are compared with the histograms of the h4 it stored), --dff N.
#define LAROSA_PHASE_CLOCK 1
#include "fused.hip"
#include "gemv.hip"
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <cmath>
#include <vector>
#include <algorithm>
#include <numeric>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1); } } while (0)
using namespace larosa;
namespace larosa { int batched_tokens_per_group(int, bool) { return 0; } }

static inline uint32_t hashu(uint32_t x) { x ^= x >> 15; x *= 2246822519u; x ^= x >> 13; x *= 3266489917u; x ^= x >> 16; return x; }
static inline float wval(size_t i, unsigned seed) { uint32_t x = hashu((uint32_t)i * 2654435761u + seed); return ((x & 0xFFFF) / 65536.0f - 0.5f) * 0.07f; }
__global__ void fill_w(uint16_t* w, size_t n, unsigned seed) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, st = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += st) { uint32_t x = (uint32_t)i * 2654435761u + seed; x ^= x >> 15; x *= 2246822519u; x ^= x >> 13; x *= 3266489917u; x ^= x >> 16;
    float f = ((x & 0xFFFF) / 65536.0f - 0.5f) * 0.07f; w[i] = __builtin_bit_cast(uint16_t, (_Float16)f); } }
static uint16_t f2h(float f) { _Float16 h = (_Float16)f; uint16_t b; memcpy(&b, &h, 2); return b; }
static float h2f(uint16_t b) { _Float16 h; memcpy(&h, &b, 2); return (float)h; }

struct Shape { const char* n; int d_in, d_out, K; bool side; int pair; };

int main(int argc, char** argv) {
  int g_main = 0, g_side = 0, reps = 40; const char* only = nullptr; bool hint = false; int dff = 11008;
  for (int i = 1; i < argc; ++i) {
    if (!strcmp(argv[i], "--gmain")) g_main = atoi(argv[++i]);
    else if (!strcmp(argv[i], "--gside")) g_side = atoi(argv[++i]);
    else if (!strcmp(argv[i], "--reps")) reps = atoi(argv[++i]);
    else if (!strcmp(argv[i], "--only")) only = argv[++i];
    else if (!strcmp(argv[i], "--hint")) hint = true;
    else if (!strcmp(argv[i], "--dff")) dff = atoi(argv[++i]);
  }
  Shape shapes[] = {{"qkv", 4096, 12288, 2457, false, 0}, {"qkv+ad", 4096, 12288, 2457, true, 0}, {"o", 4096, 4096, 2457, false, 0},
                    {"gu", 4096, 2 * dff, 2457, false, dff}, {"gu+ad", 4096, 2 * dff, 2457, true, dff}, {"down", dff, 4096, dff == 11008 ? 6604 : 5, false, 0}};
  unsigned* ctr; CK(hipMalloc(&ctr, 1 << 20)); CK(hipMemset(ctr, 0, 1 << 20));
  float* partial; CK(hipMalloc(&partial, 64 << 20));
  unsigned long long* dbg; CK(hipMalloc(&dbg, 2048 * kPhaseSlots * 8));
  const int nA = 6;
  std::vector<uint16_t*> As(nA);
  for (int i = 0; i < nA; ++i) { CK(hipMalloc(&As[i], 4096ull * 4096 * 2)); hipLaunchKernelGGL(fill_w, dim3(4096), dim3(256), 0, 0, As[i], 4096ull * 4096, 1000u + i); }
  double total_ev = 0, total_span = 0;
  for (auto& sh : shapes) {
    if (only && strcmp(only, sh.n)) continue;
    const size_t wn = (size_t)sh.d_in * sh.d_out, wb = wn * 2;
    const int nset = (int)std::min<size_t>(8, std::max<size_t>(3, (700u << 20) / wb + 1));
    std::vector<uint16_t*> Ws(nset);
    for (int i = 0; i < nset; ++i) { CK(hipMalloc(&Ws[i], wb)); hipLaunchKernelGGL(fill_w, dim3(4096), dim3(256), 0, 0, Ws[i], wn, 7u + i); }
    // heavy-tailed activation vector, rounded to f16
    std::vector<uint16_t> hb(sh.d_in); std::vector<float> hv(sh.d_in);
    for (int i = 0; i < sh.d_in; ++i) { uint32_t x = hashu(i * 7919u + 13u), y = hashu(i * 104729u + 7u);
      float u1 = ((x & 0xFFFFFF) + 1) / 16777217.0f, u2 = (y & 0xFFFFFF) / 16777216.0f;
      float z = sqrtf(-2.f * logf(u1)) * cosf(6.2831853f * u2) * powf((float)(i % 977 + 1), -0.4f) * 3.0f;
      hb[i] = f2h(z); hv[i] = h2f(hb[i]); }
    uint16_t* src; CK(hipMalloc(&src, sh.d_in * 2)); CK(hipMemcpy(src, hb.data(), sh.d_in * 2, hipMemcpyHostToDevice));
    uint16_t* y; CK(hipMalloc(&y, sh.d_out * 2)); CK(hipMemset(y, 0, sh.d_out * 2));
    uint16_t* pair_out; CK(hipMalloc(&pair_out, 32768 * 2));
    unsigned* hist; CK(hipMalloc(&hist, kHistWords * 4)); CK(hipMemset(hist, 0, kHistWords * 4));
    uint16_t* sy; CK(hipMalloc(&sy, 4096 * 2));
    int32_t* idx_out; CK(hipMalloc(&idx_out, sh.K * 4));
    FusedArgs a{}; a.g.y = y; a.g.d_in = sh.d_in; a.g.d_out = sh.d_out; a.g.K = sh.K; a.g.B = 1;
    a.pair_cols = sh.pair; a.pair_out = sh.pair ? pair_out : nullptr;
    int mg = g_main, sg = g_side;
    if (sh.side && !mg) mg = 256;
    if (sh.side && !sg) sg = 192;
    GemvPlan p = plan_fused(sh.d_out, sh.K, mg, sh.pair);
    a.g.chunk = p.chunk; a.g.wps = p.wps; a.g.G = p.G; a.g.nstrips = p.nstrips; a.g.counters = ctr; a.g.partial = partial;
    a.src_mode = kSrcPlain; a.src = src; a.d_q = sh.d_in; a.d_kv = sh.d_in; a.head_dim = 128; a.group = 1; a.idx_out = idx_out;
    const bool is_down = !strcmp(sh.n, "down");
    if (hint && sh.pair) a.hist_out = hist, a.hist_weight = 1;
    if (hint && is_down) {
      std::vector<unsigned> hh(kHistWords, 0u);
      for (int i = 0; i < sh.d_in; ++i) { unsigned key = hb[i] & 0x7FFF; hh[key >> 7]++; hh[kHistCoarse + key]++; }
      CK(hipMemcpy(hist, hh.data(), kHistWords * 4, hipMemcpyHostToDevice));
      a.hist_in = hist;
    }
    if (sh.side) {
      GemvPlan ps = plan_gemv(4096, 4096, sg);
      a.side.h = src; a.side.y = sy; a.side.d_in = 4096; a.side.d_out = 4096; a.side.K = 4096; a.side.B = 1;
      a.side.chunk = ps.chunk; a.side.wps = ps.wps; a.side.G = ps.G; a.side.nstrips = ps.nstrips;
      a.side.counters = ctr + (size_t)p.nstrips * kCounterStride; a.side.partial = partial + p.partial_floats;
      a.side_G = ps.G;
    }
    const int Gtot = p.G + a.side_G;
    unsigned long long* null = nullptr;
    CK(hipMemcpyToSymbol(HIP_SYMBOL(larosa_phase_clock), &null, sizeof(null)));
    for (int r = 0; r < 6; ++r) { a.g.W = Ws[r % nset]; a.side.W = sh.side ? As[r % nA] : nullptr; CK(launch_fused(a, false, 0)); }
    CK(hipDeviceSynchronize());
    hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    CK(hipEventRecord(e0, 0));
    for (int r = 0; r < reps; ++r) { a.g.W = Ws[r % nset]; a.side.W = sh.side ? As[r % nA] : nullptr; CK(launch_fused(a, false, 0)); }
    CK(hipEventRecord(e1, 0)); CK(hipDeviceSynchronize());
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    // phase clocks, three launches
    CK(hipMemcpyToSymbol(HIP_SYMBOL(larosa_phase_clock), &dbg, sizeof(dbg)));
    double ph[kPhaseSlots] = {0}, mx[kPhaseSlots] = {0}, span = 0; const int nph = 3; std::vector<unsigned long long> hlast;
    for (int r = 0; r < nph; ++r) {
      CK(hipMemset(dbg, 0, 2048 * kPhaseSlots * 8));
      if (a.hist_out) CK(hipMemset(hist, 0, kHistWords * 4));
      a.g.W = Ws[(r + 1) % nset]; a.side.W = sh.side ? As[(r + 2) % nA] : nullptr; CK(launch_fused(a, false, 0)); CK(hipDeviceSynchronize());
      std::vector<unsigned long long> h((size_t)Gtot * kPhaseSlots); CK(hipMemcpy(h.data(), dbg, h.size() * 8, hipMemcpyDeviceToHost));
      hlast = h;
      unsigned long long t0 = ~0ull, te = 0;
      for (int g = 0; g < Gtot; ++g) for (int i = 0; i < kPhaseSlots; ++i) { unsigned long long v = h[(size_t)g * kPhaseSlots + i]; if (v) { t0 = std::min(t0, v); te = std::max(te, v); } }
      span += (te - t0) * 0.01 / nph;
      for (int i = 0; i < kPhaseSlots; ++i) { double s = 0, m = 0; int n = 0;
        for (int g = a.side_G; g < Gtot; ++g) { unsigned long long v = h[(size_t)g * kPhaseSlots + i]; if (v) { double t = (v - t0) * 0.01; s += t; m = std::max(m, t); ++n; } }
        if (n) { ph[i] += s / n / nph; mx[i] = std::max(mx[i], m); } }
    }
    // host check: Top-K by sort, 48 sampled columns in fp64
    std::vector<int> ord(sh.d_in); std::iota(ord.begin(), ord.end(), 0);
    std::stable_sort(ord.begin(), ord.end(), [&](int x, int yy) { return (hb[x] & 0x7FFF) > (hb[yy] & 0x7FFF); });
    std::vector<int> keep(ord.begin(), ord.begin() + sh.K); std::sort(keep.begin(), keep.end());
    std::vector<int> gi(sh.K); CK(hipMemcpy(gi.data(), idx_out, sh.K * 4, hipMemcpyDeviceToHost));
    const bool idx_ok = gi == keep;
    std::vector<uint16_t> yb(sh.d_out); CK(hipMemcpy(yb.data(), y, sh.d_out * 2, hipMemcpyDeviceToHost));
    const unsigned seed_last = 7u + ((nph) % nset);   // weight set of the last phase launch
    double err = 0, nrm = 0;
    for (int s = 0; s < 48; ++s) { const int col = (int)((size_t)s * 2654435761u % sh.d_out);
      double ref = 0; for (int t = 0; t < sh.K; ++t) { const int j = keep[t]; ref += (double)hv[j] * (double)h2f(f2h(wval((size_t)j * sh.d_out + col, seed_last))); }
      const double got = h2f(yb[col]); err += (got - ref) * (got - ref); nrm += ref * ref; }
    if (a.hist_out) {
      std::vector<uint16_t> po(sh.pair); CK(hipMemcpy(po.data(), pair_out, sh.pair * 2, hipMemcpyDeviceToHost));
      std::vector<unsigned> hh(kHistWords, 0u), gh(kHistWords);
      for (int i = 0; i < sh.pair; ++i) { unsigned key = po[i] & 0x7FFF; hh[key >> 7]++; hh[kHistCoarse + key]++; }
      CK(hipMemcpy(gh.data(), hist, kHistWords * 4, hipMemcpyDeviceToHost));
      long bad = 0, tot = 0; for (int i = 0; i < kHistWords; ++i) { bad += gh[i] != hh[i]; if (i < kHistCoarse) tot += gh[i]; }
      printf("        histograms of pair_out: %ld words differ, coarse total %ld (want %d)\n", bad, tot, sh.pair);
    }
    const double us = ms * 1000.0 / reps, bytes = (double)sh.K * sh.d_out * 2 + (sh.side ? 4096.0 * 4096 * 2 : 0);
    printf("%-7s G %d+%d chunk %d  event %6.2f us (%4.2f TB/s)  span %6.2f | idx %s relL2(48 cols) %.1e\n", sh.n, p.G, a.side_G, p.chunk, us, bytes / us * 1e-6, span,
           idx_ok ? "ok" : "WRONG", sqrt(err / nrm));
    printf("        avg: start %.2f vec %.2f sel %.2f emit %.2f bar %.2f (list at %.2f) | strm %.2f fin %.2f   max: list %.2f strm %.2f fin %.2f\n",
           ph[0], ph[1] - ph[0], ph[2] - ph[1], ph[3] - ph[2], ph[4] - ph[3], ph[4], ph[5], ph[6], mx[4], mx[5], mx[6]);
    // hand-off of the workgroup that ends last: stamps 5 (stream end), 7 (LDS sum done), 8 (partial stored), 9 (arrival known), 10 (partials read), 6 (end)
    { int gl = -1; unsigned long long best = 0; for (int g = a.side_G; g < Gtot; ++g) { unsigned long long v = hlast[(size_t)g * kPhaseSlots + 6]; if (v > best) { best = v; gl = g; } }
      if (gl >= 0) { const unsigned long long* r = &hlast[(size_t)gl * kPhaseSlots];
        printf("        last WG %d: strm->lds %.2f ->stored %.2f ->arrived %.2f ->read %.2f ->end %.2f (finisher %s)\n", gl, (r[7] - r[5]) * 0.01, (r[8] - r[7]) * 0.01, (r[9] - r[8]) * 0.01,
               r[10] ? (r[10] - r[9]) * 0.01 : 0.0, (r[6] - (r[10] ? r[10] : r[9])) * 0.01, r[10] ? "yes" : "no"); }
      double a78 = 0, a89 = 0, a57 = 0; int n = 0; for (int g = a.side_G; g < Gtot; ++g) { const unsigned long long* r = &hlast[(size_t)g * kPhaseSlots]; if (r[8] && r[9]) { a57 += (r[7] - r[5]) * 0.01; a78 += (r[8] - r[7]) * 0.01; a89 += (r[9] - r[8]) * 0.01; ++n; } }
      if (n) printf("        all WGs avg: strm->lds %.2f store+wait %.2f atomic+barrier %.2f\n", a57 / n, a78 / n, a89 / n); }
    fflush(stdout);
    total_ev += us; total_span += span;
    for (auto w : Ws) CK(hipFree(w)); CK(hipFree(src)); CK(hipFree(y)); CK(hipFree(pair_out)); CK(hipFree(sy)); CK(hipFree(idx_out)); CK(hipFree(hist));
  }
  printf("sum of event times %.2f us, of spans %.2f us\n", total_ev, total_span);
  return 0;
}
