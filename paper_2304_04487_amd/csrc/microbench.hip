// llma_microbench: stand-alone measurements behind the design decisions of the decoding-step kernels
// (LLaMA-7B shapes, synthetic weights; nothing here is on the library's path):
//
//   llma_microbench shapes     the tile-K GEMM of a decoding step over its launch shapes (feature tiles
//                              per workgroup x waves) next to a plain streaming read of the same bytes
//   llma_microbench timeline   per-wave time stamps inside one tile-K launch: kernel entry, first
//                              operands arrived, end of the K loop, end of the epilogue
//   llma_microbench side-branch  the four GEMMs of a layer back to back on one stream, with and without a second stream that
//                              reads the first megabytes of the NEXT GEMM's weights while the current one runs (what a
//                              side branch of a captured graph would do)
//   llma_microbench lo8         the one-byte lo plane of the K/V cache: the library's encode / widen helpers on 3462 values
//                              against a host model of OCP fp8 e4m3 (round to nearest even, subnormals, saturation)
//   llma_microbench two-phase  two weight-streaming phases (gate/up then down, ...) as two kernels back
//                              to back, as one kernel, and as one kernel with a grid-wide barrier between
//                              the phases (with / without agent-scope fences, with / without requesting the
//                              second phase's first blocks before the barrier).  Every wait is bounded.
//
// The GEMM kernels are the library's own (this file includes their source).
#include <hip/hip_runtime.h>
#define TR_WG 2048
__device__ unsigned long long tk_trace[TR_WG * 16 * 4];
// per wave (lane 0): slot 0 kernel entry; 1 after the wave's first MFMA batch; 2 end of the K loop; 3 end of the epilogue
#define TK_STAMP(slot) tk_trace[((size_t)(blockIdx.x % TR_WG) * 16 + (threadIdx.x >> 6)) * 4 + (slot)] = wall_clock64()
#define TK_TRACE_0 int tk_seen = 0; if ((threadIdx.x & 63) == 0) TK_STAMP(0)
#define TK_TRACE_1 if ((threadIdx.x & 63) == 0 && !tk_seen) { tk_seen = 1; TK_STAMP(1); }
#define TK_TRACE_2 if ((threadIdx.x & 63) == 0) TK_STAMP(2)
#define TK_TRACE_3 if ((threadIdx.x & 63) == 0) TK_STAMP(3)
// panel GEMM (batched steps): per wave and chunk of the K loop: 0 chunk start, 1 MFMAs issued, 2 next chunk's
// activations parked in LDS, 3 past the chunk barrier; chunk 63: 0 kernel entry, 1 first chunk staged, 2 partial sums written
#define PN_WG 1024
__device__ unsigned long long pn_trace[(size_t)PN_WG * 8 * 64 * 4];
#ifdef MICROBENCH_TIMELINE
#define TK_TRACE(slot) TK_TRACE_##slot
#define PN_TRACE(slot, chunk) if ((threadIdx.x & 63) == 0 && (chunk) < 64 && blockIdx.y * gridDim.x + blockIdx.x < PN_WG) \
    pn_trace[(((size_t)(blockIdx.y * gridDim.x + blockIdx.x) * 8 + (threadIdx.x >> 6)) * 64 + (chunk)) * 4 + (slot)] = wall_clock64()
#endif
#include "kernels_bf16.hip"

#include <stdio.h>
#include <math.h>
#include <string.h>
#include <algorithm>
#include <vector>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)

static char *wbuf;
static const size_t W_BYTES = (size_t)6 << 30;          // weights rotate through 6 GB so that every launch streams from HBM
static hipEvent_t e0, e1;

__global__ void touch_kernel(const u32x4 *p, size_t n, unsigned *sink) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
    unsigned acc = 0;
    for (; i + 3 * stride < n; i += 4 * stride) {
        u32x4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
        acc ^= a.x ^ b.y ^ c.z ^ d.w;
    }
    for (; i < n; i += stride) acc ^= p[i].x;
    if (acc == 0x12345678u) *sink = acc;
}

// ------------------------------------------------------------------------------------------------ GEMM set-up
struct Shape { const char *name; int N, K, epi, tiles; };
static const int D = 4096, F = 11008, V = 32000, H = 32, DH = 128, MAX_SEQ = 2048;
static const Shape SHAPES[] = {{"qkv", 3 * D, D, EPI_QKV, 1}, {"o", D, D, EPI_RESID, 1}, {"gateup", F, D, EPI_SWIGLU, 2}, {"down", D, F, EPI_RESID, 1}, {"lmhead", V, D, EPI_LMHEAD, 1}};
struct Bufs { void *xh, *xl, *qh, *ql, *acth, *actl, *kh, *kl, *vh, *vl; float *h, *ssq, *gain, *pval, *cs; int *pidx, *rpos, *rslot; unsigned *sink; };
static void *zalloc(size_t b) { void *p; CK(hipMalloc(&p, b)); CK(hipMemset(p, 0, b)); return p; }
static Bufs make_bufs() {
    Bufs b;
    b.xh = zalloc(4 << 20); b.xl = zalloc(4 << 20); b.qh = zalloc(4 << 20); b.ql = zalloc(4 << 20); b.acth = zalloc(8 << 20); b.actl = zalloc(8 << 20);
    b.h = (float *)zalloc(512 * D * 4); b.ssq = (float *)zalloc(512 * 256 * 4); b.gain = (float *)zalloc(D * 4);
    b.pval = (float *)zalloc(64 * 2000 * 4); b.pidx = (int *)zalloc(64 * 2000 * 4); b.sink = (unsigned *)zalloc(64);
    b.rpos = (int *)zalloc(4096); b.rslot = (int *)zalloc(4096); b.cs = (float *)zalloc((size_t)MAX_SEQ * 64 * 2 * 4);
    const size_t kv = (size_t)H * MAX_SEQ * DH * 2;
    b.kh = zalloc(kv); b.kl = zalloc(kv); b.vh = zalloc(kv); b.vl = zalloc(kv);
    return b;
}
static GemmArgs make_args(const Shape &sh, const Bufs &b, int rows, size_t &bytes) {
    GemmPlan p = make_gemm_plan(sh.N, sh.K, sh.tiles), pdown = make_gemm_plan(D, F, 1);
    bytes = (size_t)(sh.N / 16) * sh.tiles * p.KSp * 1024;
    GemmArgs a{};
    a.plan = p; a.Xhi = (sh.K == F) ? b.acth : b.xh; a.Xlo = (sh.K == F) ? b.actl : b.xl; a.rows = rows; a.epi = sh.epi; a.split = 1;
    a.ssq_in = b.ssq; a.ssq_tiles = D / 16; a.eps = 1e-6f; a.out = sh.epi == EPI_RESID ? b.h : nullptr; a.gain = b.gain;
    a.nx_hi = b.xh; a.nx_lo = b.xl; a.nx_KSp = D / 32; a.ssq_out = b.ssq; a.act_hi = b.acth; a.act_lo = b.actl; a.act_KSp = pdown.KSp;
    a.pval = b.pval; a.pidx = b.pidx; a.n_part = V / 16; a.row_pos = b.rpos; a.row_slot = b.rslot; a.row_cs = b.cs; a.q_hi = b.qh; a.q_lo = b.ql;
    a.k_hi = b.kh; a.k_lo = b.kl; a.v_hi = b.vh; a.v_lo = b.vl; a.H = H; a.dh = DH; a.max_seq = MAX_SEQ;
    return a;
}
template <int EPI, int FT>
static float time_tilek(GemmArgs a, int waves, size_t bytes, int reps, bool one_launch_with_trace = false) {
    constexpr int TILES = (EPI == EPI_SWIGLU) ? 2 : 1;
    const size_t lds = (size_t)waves * FT * TILES * 1024 + 256;
    if (lds > 160 * 1024 || waves < FT) return -1.f;
    dim3 grid((a.plan.tasks + FT - 1) / FT), block(waves * 64);
    static std::atomic<uint64_t> done{0};
    allow_full_lds((const void *)gemm_tilek_bf16<1, EPI, true, FT>, done);
    const size_t stride = (bytes + (8 << 20)) & ~(size_t)4095;
    const int nb = (int)(W_BYTES / stride);
    for (int r = 0; r < 3; ++r) { a.W = wbuf + (size_t)(r % nb) * stride; hipLaunchKernelGGL((gemm_tilek_bf16<1, EPI, true, FT>), grid, block, lds, 0, a); }
    CK(hipDeviceSynchronize());
    if (one_launch_with_trace) reps = 1;
    CK(hipEventRecord(e0, 0));
    for (int r = 0; r < reps; ++r) { a.W = wbuf + (size_t)((r + 3) % nb) * stride; hipLaunchKernelGGL((gemm_tilek_bf16<1, EPI, true, FT>), grid, block, lds, 0, a); }
    CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1)); CK(hipGetLastError());
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    return ms / reps * 1e3f;
}

// ------------------------------------------------------------------------------------------------ shapes
#ifndef MICROBENCH_TIMELINE
static void cmd_shapes() {
    Bufs b = make_bufs();
    const int reps = 24;
    for (int rows : {1, 9})
        for (const Shape &sh : SHAPES) {
            size_t bytes; GemmArgs a = make_args(sh, b, rows, bytes);
            if (rows == 1) {
                const size_t n16 = bytes / 16, stride = (bytes + (8 << 20)) & ~(size_t)4095; const int nb = (int)(W_BYTES / stride);
                for (int r = 0; r < 3; ++r) hipLaunchKernelGGL(touch_kernel, dim3(512), dim3(256), 0, 0, (const u32x4 *)(wbuf + (size_t)(r % nb) * stride), n16, b.sink);   // (first touches)
                CK(hipDeviceSynchronize()); CK(hipEventRecord(e0, 0));
                for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(touch_kernel, dim3(512), dim3(256), 0, 0, (const u32x4 *)(wbuf + (size_t)(r % nb) * stride), n16, b.sink);
                CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1)); float ms; CK(hipEventElapsedTime(&ms, e0, e1));
                printf("%-7s %6.1f MB plain streaming read (512 x 256 threads): %7.2f us %6.0f GB/s\n", sh.name, bytes / 1e6, ms / reps * 1e3, bytes / (ms / reps * 1e-3) / 1e9);
            }
            auto rep = [&](int ft, int waves, float us) {
                if (us >= 0) printf("%-7s rows %d  %d tile(s) per workgroup, %2d waves, %4d workgroups: %7.2f us %6.0f GB/s\n", sh.name, rows, ft, waves, (a.plan.tasks + ft - 1) / ft, us, bytes / (us * 1e-6) / 1e9);
            };
            for (int waves : {8, 16}) {
                switch (sh.epi) {
                    case EPI_QKV: rep(1, waves, time_tilek<EPI_QKV, 1>(a, waves, bytes, reps)); rep(3, waves, time_tilek<EPI_QKV, 3>(a, waves, bytes, reps)); break;
                    case EPI_RESID: rep(1, waves, time_tilek<EPI_RESID, 1>(a, waves, bytes, reps)); rep(2, waves, time_tilek<EPI_RESID, 2>(a, waves, bytes, reps)); break;
                    case EPI_SWIGLU: rep(1, waves, time_tilek<EPI_SWIGLU, 1>(a, waves, bytes, reps)); rep(2, waves, time_tilek<EPI_SWIGLU, 2>(a, waves, bytes, reps)); break;
                    default: rep(1, waves, time_tilek<EPI_LMHEAD, 1>(a, waves, bytes, reps)); rep(3, waves, time_tilek<EPI_LMHEAD, 3>(a, waves, bytes, reps)); break;
                }
            }
        }
}
#endif

// ------------------------------------------------------------------------------------------------ timeline
#ifdef MICROBENCH_TIMELINE
template <int EPI, int FT>
static void timeline_one(const Shape &sh, const Bufs &b, int rows, int waves) {
    size_t bytes; GemmArgs a = make_args(sh, b, rows, bytes);
    const int G = (a.plan.tasks + FT - 1) / FT;
    const float us = time_tilek<EPI, FT>(a, waves, bytes, 1, true);
    std::vector<unsigned long long> t((size_t)TR_WG * 16 * 4);
    CK(hipMemcpyFromSymbol(t.data(), HIP_SYMBOL(tk_trace), t.size() * 8));
    auto at = [&](int g, int w, int sl) { return t[((size_t)g * 16 + w) * 4 + sl]; };
    unsigned long long t0 = ~0ull, tend = 0;
    for (int g = 0; g < G; ++g) for (int w = 0; w < waves; ++w) { t0 = std::min(t0, at(g, w, 0)); tend = std::max(tend, at(g, w, 2)); }
    for (int g = 0; g < G; ++g) tend = std::max(tend, at(g, 0, 3));
    printf("%s, %d row(s), %d tile(s) per workgroup, %d waves, %d workgroups: event pair %.2f us, first wave entry -> last epilogue end %.2f us (100 MHz clock)\n",
           sh.name, rows, FT, waves, G, us, (tend - t0) * 0.01);
    const char *nm[4] = {"entry", "first operands", "K loop end", "epilogue end"};
    for (int sl = 0; sl < 4; ++sl) {
        std::vector<double> v;
        for (int g = 0; g < G; ++g) for (int w = 0; w < (sl == 3 ? 1 : waves); ++w) v.push_back((at(g, w, sl) - t0) * 0.01);
        std::sort(v.begin(), v.end()); const size_t n = v.size();
        printf("   %-15s min %6.2f  p10 %6.2f  p50 %6.2f  p90 %6.2f  max %6.2f us\n", nm[sl], v[0], v[n / 10], v[n / 2], v[n * 9 / 10], v[n - 1]);
    }
}
// one split-K launch of the panel GEMM with `rows` rows: where the time of a workgroup goes
static void timeline_panel(const Shape &sh, const Bufs &b, int rows, float *part, float *rstd) {
    size_t bytes; GemmArgs a = make_args(sh, b, rows, bytes);
    a.ksplit = a.plan.n_split; a.part = part; a.rstd_in = rstd;
    const size_t stride = (bytes + (8 << 20)) & ~(size_t)4095;
    for (int r = 0; r < 3; ++r) { a.W = wbuf + (size_t)r * stride; launch_gemm_panel_bf16(a, 0); }
    CK(hipDeviceSynchronize());
    std::vector<unsigned long long> t((size_t)PN_WG * 8 * 64 * 4, 0);
    CK(hipMemcpyToSymbol(HIP_SYMBOL(pn_trace), t.data(), t.size() * 8));
    a.W = wbuf + (size_t)3 * stride;
    CK(hipEventRecord(e0, 0)); launch_gemm_panel_bf16(a, 0); CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1)); CK(hipGetLastError());
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    CK(hipMemcpyFromSymbol(t.data(), HIP_SYMBOL(pn_trace), t.size() * 8));
    auto at = [&](int g, int w, int ch, int sl) { return t[(((size_t)g * 8 + w) * 64 + ch) * 4 + sl]; };
    unsigned long long t0 = ~0ull;
    int G = 0;
    for (int g = 0; g < PN_WG; ++g) if (at(g, 0, 63, 0)) { G = g + 1; t0 = std::min(t0, at(g, 0, 63, 0)); }
    printf("%s, %d rows, %d K ranges: %d workgroups traced, event pair around panel + finishing kernel %.2f us\n", sh.name, rows, a.ksplit, G, ms * 1e3);
    std::vector<double> entry, staged, done, mf, park, bar, nch;
    for (int g = 0; g < G; ++g)
        for (int w = 0; w < 8; ++w) {
            entry.push_back((at(g, w, 63, 0) - t0) * 0.01); staged.push_back((at(g, w, 63, 1) - at(g, w, 63, 0)) * 0.01);
            done.push_back((at(g, w, 63, 2) - t0) * 0.01);
            int n = 0;
            for (int ch = 0; ch < 63 && at(g, w, ch, 3); ++ch, ++n) {
                mf.push_back((at(g, w, ch, 1) - at(g, w, ch, 0)) * 0.01); park.push_back((at(g, w, ch, 2) - at(g, w, ch, 1)) * 0.01);
                bar.push_back((at(g, w, ch, 3) - at(g, w, ch, 2)) * 0.01);
            }
            nch.push_back(n);
        }
    auto show = [&](const char *nm, std::vector<double> &v) {
        std::sort(v.begin(), v.end()); const size_t n = v.size(); double sum = 0; for (double x : v) sum += x;
        printf("   %-34s mean %6.2f  min %6.2f  p10 %6.2f  p50 %6.2f  p90 %6.2f  max %6.2f us\n", nm, sum / n, v[0], v[n / 10], v[n / 2], v[n * 9 / 10], v[n - 1]);
    };
    show("wave entry (after first entry)", entry); show("entry -> first chunk staged", staged); show("chunks per wave", nch);
    show("chunk: start -> MFMAs issued", mf); show("chunk: park next activations", park); show("chunk: barrier", bar);
    show("partial sums written (after first entry)", done);
    // one wave in detail
    printf("   workgroup 0, wave 0, per chunk (start since entry | MFMAs | park | barrier):");
    for (int ch = 0; ch < 63 && at(0, 0, ch, 3); ++ch)
        printf("%s %5.2f|%4.2f|%4.2f|%4.2f", ch % 4 == 0 ? "\n     " : "  ", (at(0, 0, ch, 0) - at(0, 0, 63, 0)) * 0.01, (at(0, 0, ch, 1) - at(0, 0, ch, 0)) * 0.01,
               (at(0, 0, ch, 2) - at(0, 0, ch, 1)) * 0.01, (at(0, 0, ch, 3) - at(0, 0, ch, 2)) * 0.01);
    printf("\n");
}
static void cmd_panel() {
    Bufs b = make_bufs();
    float *part = (float *)zalloc((size_t)64 << 20), *rstd = (float *)zalloc(4096);
    for (int rows : {144, 272}) {
        timeline_panel(SHAPES[2], b, rows, part, rstd);
        timeline_panel(SHAPES[3], b, rows, part, rstd);
        timeline_panel(SHAPES[0], b, rows, part, rstd);
    }
}
static void cmd_timeline() {
    Bufs b = make_bufs();
    for (int rows : {1, 9}) {
        timeline_one<EPI_QKV, 3>(SHAPES[0], b, rows, 16);
        timeline_one<EPI_RESID, 1>(SHAPES[1], b, rows, 8);
        timeline_one<EPI_SWIGLU, 1>(SHAPES[2], b, rows, 8);
        timeline_one<EPI_RESID, 1>(SHAPES[3], b, rows, 8);
    }
}
#endif

// ------------------------------------------------------------------------------------------------ lo8
#ifndef MICROBENCH_TIMELINE
__global__ void lo8_roundtrip_kernel(const float *in, float *out, int n) {       // n a multiple of 8
    const int i = (blockIdx.x * blockDim.x + threadIdx.x) * 8;
    if (i + 7 >= n) return;
    const float a[4] = {in[i], in[i + 1], in[i + 2], in[i + 3]}, c[4] = {in[i + 4], in[i + 5], in[i + 6], in[i + 7]};
    const u32x4 w = lo8_operand((u32x2){lo8x4(a), lo8x4(c)});                     // eight bf16 values
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        out[i + 2 * j] = __uint_as_float(w[j] << 16);
        out[i + 2 * j + 1] = __uint_as_float(w[j] & 0xffff0000u);
    }
}
static double e4m3_model(double y) {                    // OCP fp8 e4m3fn: 3 mantissa bits, spacing 2^-9 below 2^-6, largest value 448
    if (y > 448) y = 448;
    if (y < -448) y = -448;
    if (y == 0) return 0;
    int e; frexp(y, &e);
    if (e < -5) e = -5;
    double q = nearbyint(ldexp(y, 4 - e)) * ldexp(1.0, e - 4);
    return q > 448 ? 448 : (q < -448 ? -448 : q);
}
static void cmd_lo8() {
    std::vector<float> h;
    for (int e = -24; e <= 2; ++e) for (int m = 0; m < 64; ++m) { const float v = ldexpf(1.f + m / 64.f, e); h.push_back(v); h.push_back(-v); }
    for (float v : {0.f, -0.f, 1.75f, 2.f, 1e-30f, 3.f}) h.push_back(v);
    while (h.size() % 8) h.push_back(0.f);
    const int n = (int)h.size();
    float *din, *dout; CK(hipMalloc(&din, n * 4)); CK(hipMalloc(&dout, n * 4));
    CK(hipMemcpy(din, h.data(), n * 4, hipMemcpyHostToDevice));
    hipLaunchKernelGGL(lo8_roundtrip_kernel, dim3((n / 8 + 63) / 64), dim3(64), 0, 0, din, dout, n);
    CK(hipDeviceSynchronize());
    std::vector<float> d(n); CK(hipMemcpy(d.data(), dout, n * 4, hipMemcpyDeviceToHost));
    int bad = 0;
    for (int i = 0; i < n; ++i) {
        const double want = e4m3_model((double)h[i] * 256.0) / 256.0;
        if ((double)d[i] != want && bad++ < 10) printf("lo = %.9g: device %.9g, host model %.9g\n", h[i], d[i], want);
    }
    printf("lo8: %d residuals through lo8x4 + lo8_operand (fp8 e4m3 of 256 lo, widened to bf16): %d differ from the host model\n", n, bad);
    if (bad) exit(1);
}
#endif

// ------------------------------------------------------------------------------------------------ side-branch
#ifndef MICROBENCH_TIMELINE
template <int EPI, int FT>
static void launch_tilek_on(GemmArgs a, int waves, hipStream_t st) {
    constexpr int TILES = (EPI == EPI_SWIGLU) ? 2 : 1;
    const size_t lds = (size_t)waves * FT * TILES * 1024 + 256;
    static std::atomic<uint64_t> done{0};
    allow_full_lds((const void *)gemm_tilek_bf16<1, EPI, true, FT>, done);
    hipLaunchKernelGGL((gemm_tilek_bf16<1, EPI, true, FT>), dim3((a.plan.tasks + FT - 1) / FT), dim3(waves * 64), lds, st, a);
}
static void cmd_side_branch() {
    Bufs b = make_bufs();
    hipStream_t s0, s1;
    CK(hipStreamCreate(&s0)); CK(hipStreamCreate(&s1));                 // (default priority)
    const int L = 24, NK = 4 * L;                                        // 24 "layers" of four GEMMs, weights from rotating addresses
    std::vector<hipEvent_t> ev(NK);
    for (auto &e : ev) CK(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    size_t bytes[4]; GemmArgs args[4];
    const int order[4] = {0, 1, 2, 3};                                   // qkv, o, gate/up, down
    size_t layer_bytes = 0;
    for (int i = 0; i < 4; ++i) { args[i] = make_args(SHAPES[order[i]], b, 1, bytes[i]); layer_bytes += (bytes[i] + 4095) & ~(size_t)4095; }
    const int n_slots = (int)(W_BYTES / layer_bytes);
    auto weights = [&](int k) {                                          // kernel k of the chain -> its weights
        const int l = k / 4, i = k % 4;
        size_t off = (size_t)(l % n_slots) * layer_bytes;
        for (int j = 0; j < i; ++j) off += (bytes[j] + 4095) & ~(size_t)4095;
        return wbuf + off;
    };
    auto launch = [&](int k, hipStream_t st) {
        GemmArgs a = args[k % 4]; a.W = weights(k);
        switch (k % 4) {
            case 0: launch_tilek_on<EPI_QKV, 3>(a, 16, st); break;
            case 1: launch_tilek_on<EPI_RESID, 1>(a, 8, st); break;
            case 2: launch_tilek_on<EPI_SWIGLU, 1>(a, 8, st); break;
            default: launch_tilek_on<EPI_RESID, 1>(a, 8, st); break;
        }
    };
    for (size_t pre_mb : {(size_t)0, (size_t)4, (size_t)16, (size_t)64}) {
        float best = 1e9f;
        for (int pass = 0; pass < 3; ++pass) {
            CK(hipDeviceSynchronize());
            CK(hipEventRecord(e0, s0));
            for (int k = 0; k < NK; ++k) {
                if (pre_mb && k + 1 < NK) {                              // the side branch: starts when kernel k - 1 is done, like kernel k
                    if (k > 0) CK(hipStreamWaitEvent(s1, ev[k - 1], 0));
                    const size_t n16 = std::min(pre_mb << 20, bytes[(k + 1) % 4]) / 16;
                    hipLaunchKernelGGL(touch_kernel, dim3(64), dim3(256), 0, s1, (const u32x4 *)weights(k + 1), n16, b.sink);
                }
                launch(k, s0);
                if (pre_mb) CK(hipEventRecord(ev[k], s0));
            }
            CK(hipEventRecord(e1, s0)); CK(hipEventSynchronize(e1)); CK(hipStreamSynchronize(s1)); CK(hipGetLastError());
            float ms; CK(hipEventElapsedTime(&ms, e0, e1));
            if (pass) best = std::min(best, ms / L * 1e3f);
        }
        printf("four GEMMs of a layer at one row, %2d layers back to back, next GEMM's first %2zu MB read on a second stream: %7.2f us per layer\n", L, pre_mb, best);
    }
}
#endif

// ------------------------------------------------------------------------------------------------ two-phase
#ifndef MICROBENCH_TIMELINE
struct Bar { unsigned *cnt; unsigned *grp; unsigned *err; };
#define SPIN_LIMIT (1u << 20)
__device__ __forceinline__ void wait_ge(unsigned *p, unsigned target, unsigned *err) {      // bounded: gives up and raises err
    unsigned spins = 0;
    while (__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
        if (++spins > SPIN_LIMIT || __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
            __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
        }
        __builtin_amdgcn_s_sleep(1);
    }
}
template <bool FENCE>
__device__ __forceinline__ void grid_barrier(const Bar &b, unsigned epoch, unsigned nwg, unsigned ng) {     // two levels: ng groups
    __syncthreads();
    if (threadIdx.x == 0) {
        if (FENCE) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        const unsigned g = blockIdx.x % ng, per = nwg / ng;
        const unsigned old = __hip_atomic_fetch_add(b.grp + g * 64, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old == (epoch + 1) * per - 1) __hip_atomic_fetch_add(b.cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        wait_ge(b.cnt, (epoch + 1) * ng, b.err);
        if (FENCE) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
    __syncthreads();
}
#define PF 4   // 1 KiB blocks per batch and wave
__device__ __forceinline__ unsigned stream_region(const u32x4 *p, int nblk, u32x4 (&buf)[PF], bool preloaded) {
    unsigned acc = 0;
    if (!preloaded) {
#pragma unroll
        for (int u = 0; u < PF; ++u) buf[u] = __builtin_nontemporal_load(p + (size_t)(u < nblk ? u : nblk - 1) * 64);
    }
    for (int k = 0; k < nblk; k += PF) {
        u32x4 nxt[PF];
#pragma unroll
        for (int u = 0; u < PF; ++u) { int j = k + PF + u; j = j < nblk ? j : nblk - 1; nxt[u] = __builtin_nontemporal_load(p + (size_t)j * 64); }
#pragma unroll
        for (int u = 0; u < PF; ++u) acc ^= buf[u].x ^ buf[u].y ^ buf[u].z ^ buf[u].w;
#pragma unroll
        for (int u = 0; u < PF; ++u) buf[u] = nxt[u];
    }
    return acc;
}
__device__ __forceinline__ const u32x4 *wave_region(const u32x4 *base, size_t nblk_total, int &nblk) {
    const int nw = gridDim.x * (blockDim.x >> 6), w = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    const size_t b0 = nblk_total * w / nw, b1 = nblk_total * (w + 1) / nw;
    nblk = (int)(b1 - b0);
    return base + b0 * 64 + (threadIdx.x & 63);
}
__global__ __launch_bounds__(1024) void stream1(const u32x4 *A, size_t nA, unsigned *sink) {
    int n; const u32x4 *p = wave_region(A, nA, n);
    u32x4 buf[PF];
    const unsigned acc = n > 0 ? stream_region(p, n, buf, false) : 0;
    if (acc == 0x12345678u) *sink = acc;
}
// MODE 0: no barrier; 1: barrier; 2: barrier, the second phase's first batch requested before it
template <int MODE, bool FENCE>
__global__ __launch_bounds__(1024) void stream2(const u32x4 *A, size_t nA, const u32x4 *B, size_t nB, Bar b, unsigned epoch,
                                                unsigned *act, unsigned *stale, unsigned *sink) {
    int n; const u32x4 *p = wave_region(A, nA, n);
    u32x4 buf[PF];
    unsigned acc = n > 0 ? stream_region(p, n, buf, false) : 0;
    int nb; const u32x4 *q = wave_region(B, nB, nb);
    // what a phase hands to the next one: every workgroup leaves 256 words that another workgroup reads after the barrier
    if (threadIdx.x < 256) act[blockIdx.x * 256 + threadIdx.x] = epoch * 1000003u + blockIdx.x * 256 + threadIdx.x;
    if (MODE == 2 && nb > 0) {
#pragma unroll
        for (int u = 0; u < PF; ++u) buf[u] = __builtin_nontemporal_load(q + (size_t)(u < nb ? u : nb - 1) * 64);
        loads_stay_above();
    }
    if (MODE != 0) grid_barrier<FENCE>(b, epoch, gridDim.x, 8);
    if (MODE != 0 && threadIdx.x < 256) {
        const unsigned other = (blockIdx.x + 37) % gridDim.x;
        if (act[other * 256 + threadIdx.x] != epoch * 1000003u + other * 256 + threadIdx.x) atomicAdd(stale, 1u);
    }
    acc ^= nb > 0 ? stream_region(q, nb, buf, MODE == 2) : 0;
    if (acc == 0x12345678u) *sink = acc;
}
static Bar bar; static unsigned *act, *stale, *sink; static unsigned epoch_host;
template <int MODE, bool FENCE>
static void run2(const char *name, size_t bytesA, size_t bytesB, int G, int T, int reps) {
    const size_t stride = (bytesA + bytesB + (8 << 20)) & ~(size_t)4095; const int nbuf = (int)(W_BYTES / stride);
    CK(hipMemset(stale, 0, 4));
    float best = 1e9f;
    for (int pass = 0; pass < 3; ++pass) {
        CK(hipDeviceSynchronize()); CK(hipEventRecord(e0, 0));
        for (int r = 0; r < reps; ++r) {
            const char *a = wbuf + (size_t)(r % nbuf) * stride;
            hipLaunchKernelGGL((stream2<MODE, FENCE>), dim3(G), dim3(T), 0, 0, (const u32x4 *)a, bytesA / 1024, (const u32x4 *)(a + bytesA), bytesB / 1024, bar, epoch_host, act, stale, sink);
            if (MODE != 0) ++epoch_host;
        }
        CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1)); CK(hipGetLastError());
        float ms; CK(hipEventElapsedTime(&ms, e0, e1));
        if (pass) best = std::min(best, ms / reps * 1e3f);
    }
    unsigned err, ns; CK(hipMemcpy(&err, bar.err, 4, hipMemcpyDeviceToHost)); CK(hipMemcpy(&ns, stale, 4, hipMemcpyDeviceToHost));
    printf("  %-52s %7.2f us  %5.0f GB/s   stale words read after the barrier: %u%s\n", name, best, (bytesA + bytesB) / (best * 1e-6) / 1e9, ns, err ? "   (a wait gave up)" : "");
    fflush(stdout);
    if (err) { printf("a barrier wait reached its spin limit: stopping\n"); exit(0); }
}
static void cmd_two_phase() {
    hipDeviceProp_t pr; CK(hipGetDeviceProperties(&pr, 0));
    const int n_cu = pr.multiProcessorCount, reps = 20;
    if (n_cu % 8) { printf("%d compute units: not a multiple of the barrier's 8 groups\n", n_cu); return; }
    CK(hipMalloc(&bar.cnt, 4096)); CK(hipMalloc(&bar.grp, 4096)); CK(hipMalloc(&bar.err, 4096)); CK(hipMemset(bar.err, 0, 4096));
    act = (unsigned *)zalloc(2048 * 256 * 4); stale = (unsigned *)zalloc(4096); sink = (unsigned *)zalloc(4096);
    struct { const char *name; size_t a, b; } cases[] = {{"gate/up 180.4 MB then down 90.2 MB", 180355072, 90177536}, {"K/V of 1664 positions 54.5 MB then O 33.6 MB", 54525952, 33554432},
                                                         {"down 90.2 MB then QKV 100.7 MB", 90177536, 100663296}};
    struct { int wg_per_cu, T; } shapes[] = {{1, 512}, {1, 1024}, {2, 512}};
    for (auto &c : cases) {
        printf("%s\n", c.name);
        for (auto &s : shapes) {
            const int G = n_cu * s.wg_per_cu;
            int occ = 0;
            CK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, stream2<2, true>, s.T, 0));
            if (occ < s.wg_per_cu) { printf(" %d x %d threads: not co-resident\n", G, s.T); continue; }
            printf(" %d workgroups x %d threads\n", G, s.T);
            const size_t stride = (c.a + c.b + (8 << 20)) & ~(size_t)4095; const int nbuf = (int)(W_BYTES / stride);
            float best = 1e9f;
            for (int pass = 0; pass < 3; ++pass) {
                CK(hipDeviceSynchronize()); CK(hipEventRecord(e0, 0));
                for (int r = 0; r < reps; ++r) {
                    const char *a = wbuf + (size_t)(r % nbuf) * stride;
                    hipLaunchKernelGGL(stream1, dim3(G), dim3(s.T), 0, 0, (const u32x4 *)a, c.a / 1024, sink);
                    hipLaunchKernelGGL(stream1, dim3(G), dim3(s.T), 0, 0, (const u32x4 *)(a + c.a), c.b / 1024, sink);
                }
                CK(hipEventRecord(e1, 0)); CK(hipEventSynchronize(e1)); CK(hipGetLastError());
                float ms; CK(hipEventElapsedTime(&ms, e0, e1));
                if (pass) best = std::min(best, ms / reps * 1e3f);
            }
            printf("  %-52s %7.2f us  %5.0f GB/s\n", "two kernels back to back", best, (c.a + c.b) / (best * 1e-6) / 1e9);
            run2<0, false>("one kernel, no barrier (not a valid fusion: bound)", c.a, c.b, G, s.T, reps);
            CK(hipDeviceSynchronize()); CK(hipMemset(bar.cnt, 0, 4096)); CK(hipMemset(bar.grp, 0, 4096)); epoch_host = 0;
            run2<1, false>("one kernel, barrier without fences", c.a, c.b, G, s.T, reps);
            run2<1, true>("one kernel, barrier with release/acquire fences", c.a, c.b, G, s.T, reps);
            run2<2, true>("one kernel, fenced barrier, next blocks requested early", c.a, c.b, G, s.T, reps);
        }
    }
}
#endif

int main(int argc, char **argv) {
    if (!(argc > 1 && !strcmp(argv[1], "lo8"))) { CK(hipMalloc(&wbuf, W_BYTES)); CK(hipMemset(wbuf, 0x11, W_BYTES)); }   // (lo8 streams no weights)
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
#ifdef MICROBENCH_TIMELINE
    if (argc > 1 && !strcmp(argv[1], "panel")) cmd_panel();
    else cmd_timeline();
#else
    const char *cmd = argc > 1 ? argv[1] : "";
    if (!strcmp(cmd, "shapes")) cmd_shapes();
    else if (!strcmp(cmd, "two-phase")) cmd_two_phase();
    else if (!strcmp(cmd, "side-branch")) cmd_side_branch();
    else if (!strcmp(cmd, "lo8")) cmd_lo8();
    else { printf("usage: llma_microbench shapes | two-phase | side-branch | lo8      (llma_microbench_timeline for the per-wave time stamps)\n"); return 2; }
#endif
    return 0;
}
