// C ABI of the CSAT forward pass (see include/csat.h): argument checks, workspace carving and
// kernel launches.  All arithmetic of the path lives in csat_kernels.h.
#include "csat.h"
#include "csat_kernels.h"
#include "csat_ista_fused.h"
#include "csat_omp.h"
#include "csat_fwht.h"
#include "csat_gemm_big.h"
#include "csat_attention.h"
#include "csat_measure.h"
#include "csat_launch.h"
#include "csat_peaks.h"

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <thread>
#include <vector>

using namespace csat;

namespace {

// Optional per-kernel timing: when enabled, a pair of HIP events brackets every launch on the
// caller's stream; csat_profile_read sums the elapsed times per kernel id.
struct Profiler {
    struct Span { int kid; hipEvent_t a, b; };
    bool on = false;
    std::vector<Span> spans;
    void begin(int kid, hipStream_t st) {
        if (!on) return;
        Span s{kid, nullptr, nullptr};
        if (hipEventCreate(&s.a) != hipSuccess || hipEventCreate(&s.b) != hipSuccess) return;
        (void)hipEventRecord(s.a, st);      // profiling is best effort: a failed record shows up as a failed read
        spans.push_back(s);
    }
    void end(hipStream_t st) {
        if (on && !spans.empty()) (void)hipEventRecord(spans.back().b, st);
    }
    void clear() {
        for (auto& s : spans) { (void)hipEventDestroy(s.a); (void)hipEventDestroy(s.b); }
        spans.clear();
    }
};

// Kernel-selection overrides (csat_set_option).  All zero = the library's own choices; a call's
// results and workspace needs never depend on anything but its arguments and these.
struct Options {
    int v[CSAT_OPT_COUNT] = {};
    int operator[](int k) const { return v[k]; }
};

struct Context {
    uint32_t magic;
    Profiler prof;
    Options opt;
    int decoder_kernel = -1;     // what the last decoder call on this context launched (csat_profile_decoder_kernel)
};
constexpr uint32_t kMagic = 0x43534154u;   // "CSAT"

// Options of the call in progress on this thread (set by OptionScope at the top of every entry point
// that launches kernels; the defaults otherwise, e.g. in the host-only size queries).
const Options kDefaultOptions{};
thread_local const Options* tl_opt = &kDefaultOptions;
int tl_decoder_kernel_sink = -1;
thread_local int* tl_decoder_kernel = &tl_decoder_kernel_sink;
struct OptionScope {
    const Options* prev;
    int* prev_kernel;
    explicit OptionScope(void* ctx) : prev(tl_opt), prev_kernel(tl_decoder_kernel) {
        tl_opt = &static_cast<Context*>(ctx)->opt;
        tl_decoder_kernel = &static_cast<Context*>(ctx)->decoder_kernel;
    }
    ~OptionScope() { tl_opt = prev; tl_decoder_kernel = prev_kernel; }
};

inline long long round_up(long long v, long long a) { return (v + a - 1) / a * a; }
// bf16 round trip on the host (round to nearest even), for scalars the kernels must see as the element type does
inline uint16_t f2bf_host(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
inline float bf2f_host(uint16_t h) {
    const uint32_t u = (uint32_t)h << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t esize(csat_dtype t) { return t == CSAT_BF16 ? 2 : 4; }

csat_status check_dims(const csat_dims* d) {
    if (!d) return CSAT_ERR_NULL;
    if (d->dtype != CSAT_F32 && d->dtype != CSAT_BF16) return CSAT_ERR_DTYPE;
    if (d->B <= 0 || d->H <= 0 || d->n_q <= 0 || d->n <= 0 || d->d <= 0 || d->m <= 0) return CSAT_ERR_SHAPE;
    if (d->m > d->n || (d->d % 8) != 0) return CSAT_ERR_SHAPE;
    if ((long long)d->B * d->H > 65535) return CSAT_ERR_SHAPE;
    if ((long long)d->B * d->H * d->n_q > 0x7fffffffLL) return CSAT_ERR_SHAPE;
    return CSAT_OK;
}
csat_status check_ctx(void* ctx) {
    if (!ctx) return CSAT_ERR_NULL;
    return static_cast<Context*>(ctx)->magic == kMagic ? CSAT_OK : CSAT_ERR_PARAM;
}

// Kernel-selection overrides of the call in progress (see csat_set_option in csat.h).
int decoder_choice() { const int o = (*tl_opt)[CSAT_OPT_DECODER]; return o == 1 || o == 2 ? o : 0; }   // 1: GEMM pair per iteration; 2: fused wherever it fits
int gemm_raster_choice() { return ((*tl_opt)[CSAT_OPT_RASTER] & 7) == 1 ? 0 : 1; }   // 0: column-fastest everywhere
// A row operand larger than the Infinity Cache, which a launch with XCD-owned column groups reads once per group:
// its loads carry the non-temporal hint, so that they displace less of what the launch re-reads.  Measured on
// long_video's update GEMM (A = 0.5 GB): 12.9 -> 12.2 ms per launch; a 20 MB operand (cross_modal) is better off
// cached (0.205 -> 0.219 ms with the hint), and so is the residual GEMM's 8.6 GB row operand, whose four column
// tiles share every row (7.2 -> 7.4 ms with it).  (Option bits 8 / 16: never / always, for measurements.)
bool stream_hint(long long bytes) {
    const int rx = (*tl_opt)[CSAT_OPT_RASTER];
    return (rx & 8) ? false : (rx & 16) ? true : bytes > (256LL << 20);
}
int lista_choice() { return (*tl_opt)[CSAT_OPT_LISTA] == 1 ? 1 : 0; }                // 1: element-wise epilogue
int hadamard_choice() { return (*tl_opt)[CSAT_OPT_HADAMARD] == 1 ? 1 : 0; }          // 1: iterate in LDS
int gemm_choice() { return (*tl_opt)[CSAT_OPT_GEMM] == 1 ? 1 : 0; }                  // 1: 128-wide kernel only

constexpr size_t kLdsPerWorkgroup = 160 * 1024;     // LDS of a gfx950 compute unit

// The fused decoder keeps its fp32 iterate either sparse in memory (per-lane masks: only non-zero float4
// are read and written) or dense (the whole iterate streams every iteration).  Sparse pays when the
// dense iterate is too large to stay cache-resident between iterations (short_video, 491 MB: 4.4 ms
// against 5.0 ms); on a small problem the masks only add latency (image_text, 30 MB: 0.23 ms against
// 0.19 ms).  CSAT_OPT_STATE overrides the choice (for comparing the two).
bool sparse_state(size_t dense_state_bytes) {
    const int o = (*tl_opt)[CSAT_OPT_STATE] & 3;
    if (o == 1) return false;
    if (o == 2) return true;
    return dense_state_bytes > ((size_t)128 << 20);
}

// Largest m (in 32-wide tiles) the fused decoder takes.  Its residual accumulators need 16 registers per tile: up to
// 13 tiles they fit next to the operands of the two-chunk schedule; 14 to 16 tiles fill the accumulator file and run
// on the one-chunk schedule with 128-row workgroups (a few dozen spilled registers).  That still beats the large-tile
// GEMM pair when the launch has enough 128-row groups to occupy a good part of the chip (cross_modal, m = 512,
// 154 groups: 7.3 against 9.1 ms; short_video's shape at m = 512, 600 groups: 5.2 against 8.3 ms per forward), not
// below: a group's iterations are a chain, so the launch lasts as long with 40 groups as with 150 (cross_modal's rows
// with fewer heads, forward: 39 groups 6.5 against 3.8 ms, 97 groups 7.5 against 7.2, 121 groups 7.9 against 7.6).
constexpr int kFusedMaxMT = 16;
constexpr int kFused2MaxMT = 13;
constexpr long long kFusedWideMinGroups = 128;
// Polls (about 1 us apart) a unit of the fused decoder waits for the preceding segment of its rows before it gives
// up; several seconds, against a whole launch of a few milliseconds.  CSAT_OPT_FUSED_SPIN_LIMIT overrides it.
constexpr long long kFusedSpinLimit = 1ll << 22;

// Workspace layout: one carving shared by every entry point (each uses a subset), so one
// size query serves all four calls.
struct Workspace {
    long long ldn, ldm;      // padded leading dimensions of n- and m-long operand rows
    long long ldy;           // leading dimension of the fp32 measurement rows (multiple of 32)
    int MT, nct;             // 32-wide tiles along m and n (fused decoder)
    long long rows_pad;      // rows rounded up to the fused decoder's 128-row workgroups
    bool fused;              // the fused decoder runs this shape (it applies and is not overridden)
    int* Status;     // [64]  word 0: the ISTA decoder of the last call gave up (read by csat_decoder_status)
    uint4* PhiPack;  // [nct, ~2*MT, 64]  Phi as MFMA fragments for the fused decoder
    int* FusedSync;  // [2 + rows_pad/32]  unit counter, error flag and per-group progress of the fused decoder
    uint4* Hand;     // [rows_pad/128, 4, 2*MT, 64]  residual operands handed between segments of the fused decoder
    uint8_t* Mask;   // [rows_pad/32, nct or ldn/32, 64]  non-zero masks of the sparse fp32 state (bf16 mode)
    char* PhiP;   // [m, ldn]      Phi, operand layout
    char* PhiT;   // [n, ldm]      Phi^T
    char* KT;     // [BH, d, ldn]  K^T per head
    char* VT;     // [BH, d, ldn]  V^T per head
    char* Kc;     // [BH, m, d]
    char* Vc;     // [BH, m, d]
    bf16_t* KcHL; // [BH, m, 2d]   bf16 (hi | lo) split of K~ for the score contraction (bf16 mode)
    uint4* KcPack; // [BH, MT, parts * groups, 64]  K~ as MFMA fragments for the one-kernel compressed attention (d <= 128)
    char* VcT;    // [BH, d, ldm]
    float* A;     // [rows, ldy]   compressed attention rows (the decoder's measurements), zero padded
    char* R;      // [rows, ldm]   softmax / residual operand
    float* Xs;    // [rows, ldn]   decoder state ([rows_pad, 32*nct] in fragment order when fused)
    bf16_t* Xb;   // [rows, ldn]   bf16 operand copy of the state (bf16 mode)
    char* Z;      // [rows, d]
    int split;    // > 1: the residual product runs as this many partial products along K (few output tiles)
    float* SplitP;  // [split, rows, ldm]  their outputs
    size_t bytes;
    Profiler* prof;   // never null during a call
};

Workspace carve(const csat_dims& d, char* base) {
    Workspace w{};
    const size_t e = esize(d.dtype);
    const long long BH = (long long)d.B * d.H, rows = BH * d.n_q;
    // bf16 operand rows are zero-padded to a multiple of 64 elements (the large-tile GEMM's K step)
    const long long kpad = d.dtype == CSAT_BF16 ? 64 : 8;
    w.ldn = round_up(d.n, kpad);
    w.ldm = round_up(d.m, kpad);
    w.ldy = round_up(d.m, 32);
    w.MT = (int)(w.ldy / 32);
    w.nct = (int)((d.n + 31) / 32);
    w.rows_pad = round_up(rows, 128);
    // The carving does not depend on the kernel-selection overrides: buffers that differ between the
    // fused decoder and the GEMM pair are sized for the larger of the two.
    const bool fused_ok = d.dtype == CSAT_BF16 && w.MT <= kFusedMaxMT && w.nct >= 3;
    const bool fused_pays = w.MT <= kFused2MaxMT || w.rows_pad / 128 >= kFusedWideMinGroups;
    w.fused = fused_ok && decoder_choice() != 1 && (fused_pays || decoder_choice() == 2);
    size_t off = 0;
    auto take = [&](size_t nbytes) {
        char* p = base + off;
        off += (size_t)round_up((long long)nbytes, 256);
        return p;
    };
    w.Status = (int*)take(256);
    w.PhiP = take((size_t)d.m * w.ldn * e);
    w.PhiT = take((size_t)d.n * w.ldm * e);
    w.KT = take((size_t)BH * d.d * w.ldn * e);
    w.VT = take((size_t)BH * d.d * w.ldn * e);
    w.Kc = take((size_t)BH * d.m * d.d * e);
    w.Vc = take((size_t)BH * d.m * d.d * e);
    w.KcHL = (bf16_t*)take(d.dtype == CSAT_BF16 ? (size_t)BH * d.m * d.d * 4 : 0);
    w.KcPack = (uint4*)take(d.d <= 128 ? (size_t)BH * w.MT * (d.dtype == CSAT_BF16 ? 2 * ((d.d + 15) / 16) : (d.d + 7) / 8) * 1024 : 0);
    w.VcT = take((size_t)BH * d.d * w.ldm * e);
    // (chunk count rounded up to even: the two-chunk schedule walks whole pairs, the odd one out is a zero chunk)
    w.PhiPack = (uint4*)take(fused_ok ? (size_t)((w.nct + 1) / 2 * 2) * ista_fused_set_frags(w.MT) * 1024 : 0);
    w.FusedSync = (int*)take(fused_ok ? (size_t)(2 + w.rows_pad / 32) * 4 : 0);
    w.Hand = (uint4*)take(fused_ok ? (size_t)(w.rows_pad / 128) * 4 * 2 * w.MT * 1024 : 0);
    // ldn >= 32 * nct, so the GEMM pair's mask and state sizes cover the fused decoder's
    w.Mask = (uint8_t*)take(d.dtype == CSAT_BF16 ? (size_t)(w.rows_pad / 32) * (w.ldn / 32) * 64 : 0);
    w.A = (float*)take((size_t)rows * w.ldy * 4);
    w.R = take((size_t)rows * w.ldm * e);
    w.Xs = (float*)take((size_t)w.rows_pad * w.ldn * 4);
    w.Xb = (bf16_t*)take(d.dtype == CSAT_BF16 ? (size_t)rows * w.ldn * 2 : 0);
    w.Z = take((size_t)rows * d.d * e);
    // A residual product with few 256 x 256 output tiles leaves most of the chip idle while each tile
    // walks the whole of K = n: split K so that tiles x parts comes close to the 256 CUs this is sized
    // for (parts divides the number of 64-wide K steps, at most 8).
    w.split = 1;
    if (d.dtype == CSAT_BF16 && rows >= 256 && w.ldm >= 128) {
        const long long tiles = ((rows + 255) / 256) * ((w.ldm + 255) / 256), ksteps = w.ldn / 64;
        for (int s = 2; s <= 8; ++s)
            if (ksteps % s == 0 && tiles * s <= 256) w.split = s;
    }
    w.SplitP = (float*)take(w.split > 1 ? (size_t)w.split * rows * w.ldm * 4 : 0);
    w.bytes = off;
    return w;
}

#define HIP_TRY(expr)                                  \
    do {                                               \
        if ((expr) != hipSuccess) return CSAT_ERR_HIP; \
    } while (0)
#define CSAT_TRY(expr)                  \
    do {                                \
        csat_status s_ = (expr);        \
        if (s_ != CSAT_OK) return s_;   \
    } while (0)

struct Timed {   // brackets the launches issued during its lifetime
    Profiler* p; hipStream_t st;
    Timed(const Workspace& w, int kid, hipStream_t s) : p(w.prof), st(s) { p->begin(kid, st); }
    ~Timed() { p->end(st); }
};

template <typename T, int BM, int BN, int WM, int WN, typename Epi>
csat_status launch_gemm(const GemmArgs& g, long long n_cover, int batch, const Epi& epi, hipStream_t st) {
    // n_cover >= N: columns the epilogue must visit (pads included)
    dim3 grid((unsigned)((g.M + BM - 1) / BM), (unsigned)((n_cover + BN - 1) / BN), (unsigned)batch);
    hipLaunchKernelGGL((gemm_nt_kernel<T, BM, BN, WM, WN, Epi>), grid, dim3(256), 0, st, g, epi);
    HIP_TRY(hipGetLastError());
    return CSAT_OK;
}

template <typename Epi, int WM, int WN, int KS>
csat_status launch_gemm_big_shape(const GemmArgs& g, long long n_cover, int batch, const Epi& epi, hipStream_t st) {
    using S = BigGemmShape<Epi, WM, WN, KS>;
    HIP_TRY(hipFuncSetAttribute((const void*)gemm_nt_bf16_big_kernel<Epi, WM, WN, KS>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)S::kLdsBytes));
    const long long tm = (g.M + S::kRowsA - 1) / S::kRowsA, tn = (n_cover + S::kRowsB - 1) / S::kRowsB;
    GemmArgs gt = g;
    gt.a_kwrap = (int)tn;     // column tiles: the kernel walks a 1-D grid
    gt.raster = (tn <= 8 && batch == 1 && gemm_raster_choice() != 0) ? 1 : 0;
    // many column tiles, a multiple of 8: each XCD keeps a few column tiles' operand in its L2 (see the kernel)
    if (const int rx = (*tl_opt)[CSAT_OPT_RASTER], ro = rx & 7; tn >= 16 && tn % 8 == 0 && batch == 1 && ro != 1) {
        const int per_xcd = (int)(tn / 8);
        int cb = ro >= 2 ? 1 << (ro - 2) : 4;                  // (option values 2, 3, 4, 5: groups of 1, 2, 4, 8 for measurements)
        while (cb > 1 && per_xcd % cb != 0) cb >>= 1;
        gt.raster = 2 + (cb == 8 ? 3 : cb == 4 ? 2 : cb == 2 ? 1 : 0);
        if (stream_hint((long long)g.M * g.K * 2)) gt.raster |= kRasterStreamA;
    }
    const long long tiles = gt.raster == 1 ? (tm + 7) / 8 * 8 * tn : tm * tn;
    dim3 grid((unsigned)tiles, 1, (unsigned)batch);
    hipLaunchKernelGGL((gemm_nt_bf16_big_kernel<Epi, WM, WN, KS>), grid, dim3(S::kThreads), S::kLdsBytes, st, gt, epi);
    HIP_TRY(hipGetLastError());
    return CSAT_OK;
}

// 256 x 256 x 64 tiles, 8 wavefronts.  (A 256 x 128 x 32 shape with two workgroups per CU, meant to
// run one workgroup's epilogue under the other's main loop, measured slower on every workload.)
template <typename Epi>
csat_status launch_gemm_big(const GemmArgs& g, long long n_cover, int batch, const Epi& epi, hipStream_t st) {
    return launch_gemm_big_shape<Epi, 4, 2, 64>(g, n_cover, batch, epi, st);
}

// Big bf16 problems whose operands are zero-padded to a multiple of 64 along K (every workspace
// operand is) go to the 256x256 kernel.  Otherwise: narrow-N problems (N <= 64) waste half of a
// 128-wide tile, so they get the 64-wide one.
template <typename T>
bool use_big_gemm(const GemmArgs& g, long long n_cover) {
    if (sizeof(T) != 2) return false;
    const long long Kp = round_up(g.K, 64);
    return Kp <= g.lda && Kp <= g.ldb && g.a_kwrap == 0 && g.M >= 256 && n_cover >= 128 && gemm_choice() != 1;
}

template <typename T, typename Epi>
csat_status gemm(const GemmArgs& g, long long n_cover, int batch, const Epi& epi, hipStream_t st) {
    if constexpr (sizeof(T) == 2) {
        const long long Kp = round_up(g.K, 64);
        if (use_big_gemm<T>(g, n_cover)) {
            GemmArgs gb = g;
            gb.K = (int)Kp;
            return launch_gemm_big<Epi>(gb, n_cover, batch, epi, st);
        }
    }
    if (n_cover <= 64) return launch_gemm<T, 128, 64, 2, 2, Epi>(g, n_cover, batch, epi, st);
    return launch_gemm<T, 128, 128, 2, 2, Epi>(g, n_cover, batch, epi, st);
}

template <typename TI, typename TO>
csat_status pack_rows(const TI* src, long long lds_, TO* dst, long long ldd, long long rows, int cols, hipStream_t st) {
    long long total = rows * ldd;
    hipLaunchKernelGGL((pack_rows_kernel<TI, TO>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                       src, lds_, dst, ldd, rows, cols);
    HIP_TRY(hipGetLastError());
    return CSAT_OK;
}

template <typename T>
csat_status transpose_pack(const T* src, T* dst, long long ldd, int batch, int R, int Cc, hipStream_t st) {
    dim3 grid((unsigned)((ldd + 31) / 32), (unsigned)((Cc + 31) / 32), (unsigned)batch);
    hipLaunchKernelGGL((transpose_pack_kernel<T>), grid, dim3(32, 8), 0, st, src, (long long)R * Cc, dst, ldd,
                       (long long)Cc * ldd, R, Cc);
    HIP_TRY(hipGetLastError());
    return CSAT_OK;
}

csat_status fill_zero(void* p, size_t bytes, hipStream_t st) {   // bytes multiple of 4
    long long words = (long long)(bytes / 4);
    if (words == 0) return CSAT_OK;
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((words + 255) / 256)), dim3(256), 0, st, (uint32_t*)p, words);
    HIP_TRY(hipGetLastError());
    return CSAT_OK;
}

// ---------------------------------------------------------------------------------------
// Stage drivers on prepared operands (typed by the element type T).
// ---------------------------------------------------------------------------------------

// Operand copies of Phi: row-major padded (measurement GEMM; generic decoder's residual GEMM),
// transposed (generic decoder's update GEMM) or MFMA fragments (fused decoder).
template <typename T>
csat_status prepare_phi(const csat_dims& d, const Workspace& w, const T* Phi, bool for_measure, bool for_decoder,
                        hipStream_t st) {
    Timed tm(w, CSAT_K_LAYOUT, st);
    const bool generic = for_decoder && !w.fused;
    if (for_measure || generic) CSAT_TRY((pack_rows<T, T>(Phi, d.n, (T*)w.PhiP, w.ldn, d.m, d.n, st)));
    if (generic) CSAT_TRY(transpose_pack<T>(Phi, (T*)w.PhiT, w.ldm, 1, d.m, d.n, st));
    if constexpr (sizeof(T) == 2) {
        if (for_decoder && w.fused) {
            const int nct2 = (w.nct + 1) / 2 * 2;
            long long total = (long long)nct2 * ista_fused_set_frags(w.MT) * 64;
            hipLaunchKernelGGL(pack_phi_fragments_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                               (const bf16_t*)Phi, d.m, d.n, w.MT, nct2, w.PhiPack);
            HIP_TRY(hipGetLastError());
        }
    }
    return CSAT_OK;
}

// Whether the measurement runs as the one kernel that reads K and V as they are (csat_measure.h): bf16, d of
// one or two 64-wide tiles, one matrix for both products.
template <typename T>
bool measure_is_direct(const csat_dims& d, bool separate) {
    return sizeof(T) == 2 && !separate && (d.d == 64 || d.d == 128) && (*tl_opt)[CSAT_OPT_MEASURE] != 1;
}
// The synthesis straight from V as the caller holds it ([n, d] per head): the measurement kernel with the head's rows
// of the bf16 iterate as its row operand (csat_measure.h), no transposed copy of V.  bf16 with d = 64 or 128.
template <typename T>
bool synthesis_is_direct(const csat_dims& d) {
    return sizeof(T) == 2 && (d.d == 64 || d.d == 128) && (*tl_opt)[CSAT_OPT_SYNTHESIS] != 2;
}
// ... and whether it reads Phi as the caller holds it (rows 16-byte aligned), so that no operand copy is needed
template <typename T>
bool measure_reads_raw_phi(const csat_dims& d, bool separate) { return measure_is_direct<T>(d, separate) && d.n % 8 == 0; }

// Kc = Phi_K K, Vc = Phi V (+ transposed copy of Vc when VcT != nullptr).  vt_ready: the caller needs no transposed
// copy of V in w.VT afterwards (the one-kernel path then makes none).  w.PhiP holds Phi (= Phi_V) on
// entry and on return; a separate key matrix PhiK (raw, caller layout) borrows it for the K product.
// *kc_packed (optional) reports whether K~'s (hi | lo) fragments for the one-kernel attention were written too.
// v_packed (optional): the caller will run the one-kernel attention with its own output product; *v_packed then
// reports that the VcT buffer holds V~ as that product's fragments instead of the transpose.
template <typename T>
csat_status run_measure(const csat_dims& d, const Workspace& w, const T* K, const T* V, T* Kc, T* Vc, T* VcT,
                        bool vt_ready, bool split_k, hipStream_t st, const T* PhiK = nullptr,
                        const T* PhiV = nullptr, bool want_v = true, bool* kc_packed = nullptr,
                        bool* v_packed = nullptr) {
    const bool separate = PhiK && PhiK != PhiV;
    const int BH = d.B * d.H;
    if (kc_packed) *kc_packed = false;
    if (v_packed) *v_packed = false;
    if constexpr (sizeof(T) == 2) {
        // one matrix for both products and d of one or two 64-wide tiles: both products in one launch, straight
        // from K and V as they are, with every copy of K~ and V~ the next stage reads (csat_measure.h)
        if (measure_is_direct<T>(d, separate)) {
            if (!vt_ready) {
                Timed tm(w, CSAT_K_LAYOUT, st);
                CSAT_TRY(transpose_pack<T>(V, (T*)w.VT, w.ldn, BH, d.n, d.d, st));
            }
            Timed tm(w, CSAT_K_MEASURE, st);
            MeasureDirectArgs a{};
            // Phi as the caller holds it where its rows are 16-byte aligned, else the zero-padded operand copy
            const bool raw = PhiV && measure_reads_raw_phi<T>(d, separate);
            a.Phi = raw ? (const bf16_t*)PhiV : (const bf16_t*)w.PhiP;
            a.ldp = raw ? d.n : w.ldn;
            a.ncols = raw ? d.n : (int)w.ldn;
            a.K = (const bf16_t*)K; a.V = (const bf16_t*)V; a.strideX = (long long)d.n * d.d;
            a.m = d.m; a.n = d.n; a.MT = w.MT;
            a.Kc = (bf16_t*)Kc;
            a.KcHL = split_k ? w.KcHL : nullptr;
            a.KcPack = split_k && kc_packed ? w.KcPack : nullptr;
            a.Vc = want_v ? (bf16_t*)Vc : nullptr;
            const bool frags = v_packed && VcT && want_v && (*tl_opt)[CSAT_OPT_MEASURE] != 2;
            a.VcT = frags ? nullptr : (bf16_t*)VcT; a.ldm = w.ldm;
            a.VPack = frags ? (uint4*)VcT : nullptr;        // (MT * 32 <= ldm: the fragments fit the transpose's buffer)
            if (frags) *v_packed = true;
            a.heads = BH;
            a.blocks_per_head = want_v ? (w.MT + 1) / 2 : (w.MT + 3) / 4;
            const dim3 grid((unsigned)(8 * ((BH + 7) / 8) * a.blocks_per_head));
            // 64 rows of K and V per step; two steps in flight, four for long contractions (measured on the five
            // workloads: 26 us either way at n = 1600, 221 against 247 us at n = 4096, 238 against 285 at n = 16384)
#define MD(DT, PD)                                                                                      \
    do {                                                                                                \
        if (want_v) hipLaunchKernelGGL((measure_direct_kernel<DT, 64, PD, true>), grid, dim3(256), 0, st, a);  \
        else hipLaunchKernelGGL((measure_direct_kernel<DT, 64, PD, false>), grid, dim3(256), 0, st, a); \
    } while (0)
            const bool deep = d.n >= 4096;
            if (d.d == 64) { if (deep) MD(2, 4); else MD(2, 2); }
            else { if (deep) MD(4, 4); else MD(4, 2); }
#undef MD
            HIP_TRY(hipGetLastError());
            if (kc_packed) *kc_packed = a.KcPack != nullptr;
            return CSAT_OK;
        }
    }
    {
        Timed tm(w, CSAT_K_LAYOUT, st);
        CSAT_TRY(transpose_pack<T>(K, (T*)w.KT, w.ldn, BH, d.n, d.d, st));
        if (!vt_ready) CSAT_TRY(transpose_pack<T>(V, (T*)w.VT, w.ldn, BH, d.n, d.d, st));
        if (VcT) CSAT_TRY(fill_zero(VcT, (size_t)BH * d.d * w.ldm * sizeof(T), st));
    }
    if (separate) {
        Timed tl(w, CSAT_K_LAYOUT, st);
        CSAT_TRY((pack_rows<T, T>(PhiK, d.n, (T*)w.PhiP, w.ldn, d.m, d.n, st)));
    }
    Timed tm(w, CSAT_K_MEASURE, st);
    GemmArgs g{w.PhiP, w.ldn, 0, w.KT, w.ldn, (long long)d.d * w.ldn, d.m, d.d, d.n, 0};
    if constexpr (sizeof(T) == 2) {
        if (split_k) {
            EpiMeasureSplit ek{(bf16_t*)Kc, w.KcHL, d.m, d.d};
            CSAT_TRY((gemm<T>(g, d.d, BH, ek, st)));
        }
    }
    if (sizeof(T) != 2 || !split_k) {
        EpiStore<T> ek{Kc, d.d, (long long)d.m * d.d, nullptr, 0, 0, 1.f, d.m, d.d};
        CSAT_TRY((gemm<T>(g, d.d, BH, ek, st)));
    }
    if (separate) CSAT_TRY((pack_rows<T, T>(PhiV, d.n, (T*)w.PhiP, w.ldn, d.m, d.n, st)));
    if (!want_v) return CSAT_OK;      // (V~ only feeds the compressed output Z: a forward without Z does not need it)
    g.Bt = w.VT;
    EpiStore<T> ev{Vc, d.d, (long long)d.m * d.d, VcT, w.ldm, (long long)d.d * w.ldm, 1.f, d.m, d.d};
    CSAT_TRY((gemm<T>(g, d.d, BH, ev, st)));
    return CSAT_OK;
}

// CUs of the current device (persistent grids and work-distribution heuristics)
int cu_count() {
    static const int n = [] {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) return 256;
        return v;
    }();
    return n;
}

// Whether the one-kernel attention keeps all of a head's K~ fragments (ns per tile of m, mt tiles) in LDS and all
// score tiles of a row block in registers: one sweep over m instead of two.
bool attention_single_sweep(int mt, int ns) {
    return mt <= 16 && (size_t)attention_mtp(mt, true) * ns * 1024 <= (size_t)kAttnMaxLdsBytes;
}

// ... and whether V~'s fragments for the kernel's own output product (bf16, d = 64 or 128, K~ as the (hi | lo)
// pair) fit into LDS next to K~'s
bool attention_packed_v_fits(int mt, int d) {
    const int ns = 2 * (d / 16);
    return attention_single_sweep(mt, ns) && (size_t)attention_mtp(mt, true) * (ns + d / 16) * 1024 <= (size_t)kAttnLdsBytes;
}

// Compressed attention in one kernel (csat_attention.h; d <= 128) behind a small kernel that packs K~ as
// MFMA fragments.  Ksrc: K~ rows [BH][m][kparts * d] (the plain matrix, or the bf16 (hi | lo) pair).
// A may be null when only Z is wanted.
template <typename T>
csat_status launch_attention_fused(const csat_dims& d, const Workspace& w, const T* Q, const T* Ksrc, int kparts,
                                   const T* VcT, float* A, long long ldA, T* P, T* Z, T* ZT, hipStream_t st,
                                   bool kc_packed = false, bool v_packed = false, bool a_tiled = false) {
    constexpr int GK = sizeof(T) == 2 ? 16 : 8;          // contraction depth of one fragment
    const int BH = d.B * d.H;
    AttentionArgs a{};
    a.ng = (d.d + GK - 1) / GK;
    a.ns = kparts * a.ng;
    a.Q = Q; a.strideQ = (long long)d.n_q * d.d;
    a.Kf = w.KcPack;
    // (fragments of V~ only come from the one-kernel measurement: bf16, d = 64 or 128; ZT is not produced from them)
    a.VcT = v_packed ? nullptr : VcT; a.ldv = w.ldm; a.strideV = (long long)d.d * w.ldm;
    a.Vf = v_packed ? (const uint4*)VcT : nullptr;
    a.A = A; a.ldA = ldA; a.a_tiled = a_tiled ? 1 : 0;
    a.P = P; a.ldP = w.ldm;
    a.Z = Z;
    a.ZT = ZT; a.ldT = sizeof(T) == 2 ? 2 * w.ldn : w.ldn; a.strideT = (long long)d.d * a.ldT;
    a.n_q = d.n_q; a.m = d.m; a.d = d.d;
    a.scale_log2e = 1.4426950408889634f / sqrtf((float)d.d);
    a.tiles_per_head = (d.n_q + 31) / 32;
    const int mt = w.MT;
    const bool single = attention_single_sweep(mt, a.ns);
    // Rounds of one row tile per wavefront: with all of K~ in LDS a workgroup amortises its staging over several
    // rounds; take the count that needs the fewest passes of the grid over the chip (ties: fewer rounds).
    const int nw = attention_waves(attention_mtp(mt, single), v_packed ? 2 : 0);
    a.rounds = 1;
    if (single) {
        const int cus = cu_count();
        long long best = -1;
        for (int r = 1; r <= 8; ++r) {
            const long long wgs = (long long)BH * ((a.tiles_per_head + nw * r - 1) / (nw * r));
            const long long cost = (wgs + cus - 1) / cus * (4 * r + 1);      // + 1: the staging, about a quarter of a round
            if (best < 0 || cost < best) { best = cost; a.rounds = r; }
        }
    }
    a.wg_per_head = (a.tiles_per_head + nw * a.rounds - 1) / (nw * a.rounds);
    // LDS for all the tiles the kernel instance holds (slots of tiles beyond m are zeroed, not skipped)
    const int mtp = attention_mtp(mt, single);
    size_t lds_bytes = (size_t)mtp * a.ns * 1024;
    a.v_lds = -1;
    if (a.Vf) {      // V~'s fragments next to K~'s (single sweep; the caller made sure the CU's LDS holds both)
        const size_t vbytes = (size_t)mtp * (d.d / 16) * 1024;
        if (!single || lds_bytes + vbytes > (size_t)kAttnLdsBytes) return CSAT_ERR_SHAPE;
        a.v_lds = mtp * a.ns;
        lds_bytes += vbytes;
    }
    if (!kc_packed) {
        Timed tm(w, CSAT_K_SCORES, st);
        const long long total = (long long)BH * mt * a.ns * 64;
        hipLaunchKernelGGL((pack_kc_fragments_kernel<T>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, Ksrc,
                           (long long)kparts * d.d, d.m, d.d, kparts, mt, a.ng, w.KcPack, total);
        HIP_TRY(hipGetLastError());
    }
    const unsigned grid = (unsigned)(BH * a.wg_per_head);
    const bool want_z = Z || ZT;
    Timed tm(w, CSAT_K_SOFTMAX, st);
    if (sizeof(T) == 2) {
        // (those kernels store whole tiles only)
        if (want_z && a.Vf && ((A && (ldA % 4 != 0 || ldA < 32 * mt)) || (P && w.ldm < 32 * mt))) return CSAT_ERR_SHAPE;
        if (want_z && a.Vf) HIP_TRY(d.d == 64 ? attention_fused_launch_bf16_z2(mt, single, a, grid, lds_bytes, st)
                                              : attention_fused_launch_bf16_z3(mt, single, a, grid, lds_bytes, st));
        else HIP_TRY(want_z ? attention_fused_launch_bf16_z1(mt, single, a, grid, lds_bytes, st)
                            : attention_fused_launch_bf16_z0(mt, single, a, grid, lds_bytes, st));
    }
    else HIP_TRY(want_z ? attention_fused_launch_f32_z1(mt, single, a, grid, lds_bytes, st)
                        : attention_fused_launch_f32_z0(mt, single, a, grid, lds_bytes, st));
    return CSAT_OK;
}

// Whether the compressed attention runs as the one kernel: d <= 128 unless overridden; a head with fewer than 8 row
// tiles and more than 32 KB of K~ fragments cannot amortise keeping K~ in LDS (cross-attention with a short query
// side: 85 us against 44 us measured at 77 queries, m = 512) and takes the three kernels.
template <typename T>
bool attention_is_fused(const csat_dims& d, const Workspace& w, bool split_k) {
    const int attn_opt = (*tl_opt)[CSAT_OPT_ATTENTION];
    const int frag_depth = sizeof(T) == 2 ? 16 : 8;
    const bool short_side = (d.n_q + 31) / 32 < 8 &&
                            (long long)w.MT * (sizeof(T) == 2 && split_k ? 2 : 1) * ((d.d + frag_depth - 1) / frag_depth) > 32;
    return d.d <= 128 && attn_opt != 1 && (attn_opt == 2 || !short_side);
}

// A = softmax(Q Kc^T / sqrt(d)) (float, [rows, m]); P = operand copy [rows, ldm];
// Z = A Vc when Z != nullptr (needs VcT)
// ZT != nullptr (with Z possibly null): also the transposed output per head, [BH, d, ldn] in fp32 mode,
// [BH, d, 2*ldn] as a bf16 (hi | lo) pair in bf16 mode; ZT must be zeroed beforehand.
template <typename T>
csat_status run_attention(const csat_dims& d, const Workspace& w, const T* Q, const T* Kc, const T* VcT,
                          float* A, long long ldA, T* P, T* Z, bool split_k, hipStream_t st, T* ZT = nullptr,
                          bool kc_packed = false, bool v_packed = false, bool a_tiled = false) {
    const int BH = d.B * d.H;
    const long long rows = (long long)BH * d.n_q;
    const int attn_opt = (*tl_opt)[CSAT_OPT_ATTENTION];
    // With Z requested (the stage call, the column-wise reading, a caller that wants Z) and more than four tiles of m,
    // the one kernel's own output product, which reads V~ per wavefront, measured slower than a product kernel behind it
    // (short_video, stage call: 158 us in one kernel, 115 us as three kernels; image_text, three tiles: 33 against 39):
    // there the one kernel writes A~ and its operand copy, and Z comes from the product kernel below.  A~ is the same
    // whether Z is requested or not.
    // (With V~ as the product's fragments, written by the one-kernel measurement, the one kernel's own product reads
    // them with one coalesced load per MFMA and is the faster again.)
    const bool wide_z = (Z || ZT) && w.MT > 4 && attn_opt != 2 && P != nullptr && !v_packed;
    bool have_a = false;
    if (attention_is_fused<T>(d, w, split_k)) {
        const bool hl = sizeof(T) == 2 && split_k;                 // contract against the (hi | lo) pair of K~
        const T* Ksrc = hl ? (const T*)w.KcHL : Kc;
        const bool packed = kc_packed && hl;
        if (!wide_z) return launch_attention_fused<T>(d, w, Q, Ksrc, hl ? 2 : 1, VcT, A, ldA, P, Z, ZT, st, packed, v_packed, a_tiled);
        if (a_tiled) return CSAT_ERR_SHAPE;      // (the caller asks for tiles only where the one launch does everything)
        CSAT_TRY(launch_attention_fused<T>(d, w, Q, Ksrc, hl ? 2 : 1, VcT, A, ldA, P, (T*)nullptr, (T*)nullptr, st, packed));
        have_a = true;
    }
    if (!have_a) {      // scores with the scale fused, then the row softmax
        GemmArgs g{Q, d.d, (long long)d.n_q * d.d, Kc, d.d, (long long)d.m * d.d, d.n_q, d.m, d.d, 0};
        if (sizeof(T) == 2 && split_k) {   // [Q | Q] against [K~hi | K~lo]
            g.Bt = w.KcHL; g.ldb = 2 * d.d; g.strideB = (long long)d.m * 2 * d.d; g.K = 2 * d.d;
            g.a_kwrap = d.d / 8;
        }
        EpiStore<float> es{A, ldA, (long long)d.n_q * ldA, nullptr, 0, 0, 1.f / sqrtf((float)d.d), d.n_q, d.m};
        {
            Timed tm(w, CSAT_K_SCORES, st);
            CSAT_TRY((gemm<T>(g, d.m, BH, es, st)));
        }
        {
            Timed tm(w, CSAT_K_SOFTMAX, st);
            if (d.m <= 512)
                hipLaunchKernelGGL((softmax_rows_kernel<T, 8>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, A, ldA, rows,
                                   d.m, P, w.ldm);
            else
                hipLaunchKernelGGL((softmax_rows_kernel<T, 16>), dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st, A, ldA, rows,
                                   d.m, P, w.ldm);
            HIP_TRY(hipGetLastError());
        }
    }
    if (Z || ZT) {
        Timed tm(w, CSAT_K_OUTPUT, st);
        GemmArgs gz{P, w.ldm, (long long)d.n_q * w.ldm, VcT, w.ldm, (long long)d.d * w.ldm, d.n_q, d.d, d.m, 0};
        if constexpr (sizeof(T) == 2) {
            if (ZT) {
                EpiStoreSplitT ez{(bf16_t*)Z, d.d, (long long)d.n_q * d.d, (bf16_t*)ZT, 2 * w.ldn, (long long)d.d * 2 * w.ldn,
                                  d.n_q, d.d};
                return gemm<T>(gz, d.d, BH, ez, st);
            }
        }
        EpiStore<T> ez{Z, d.d, (long long)d.n_q * d.d, ZT, w.ldn, (long long)d.d * w.ldn, 1.f, d.n_q, d.d};
        CSAT_TRY((gemm<T>(gz, d.d, BH, ez, st)));
    }
    return CSAT_OK;
}

// Segments per group for the fused decoder: G groups of whole length take ceil(G / P) rounds on P
// CUs, units of 1/S of the length ceil(G S / P) / S; each segment start costs a pipeline refill and
// a hand-over.  `overhead`: that cost as a share of a whole-length group.  Measured on short_video (20 iterations of
// 50 chunks, 1.5 ms per group): about 30 us per hand-over, most of it the agent-scope release fence, which writes back
// the whole L2 (the state of the 32 compute units behind it): the time of about 20 chunk steps.  (Without the fences
// - results then unreliable - five segments took 3.36 ms against 3.59; handing the state over through system-scope
// accesses instead, written through and read from memory, no fences, gave the same results bit for bit and cost as
// much in every step, waiting for the write-through stores, as it saved at the hand-overs.)
int fused_segments(long long groups, int iters, int cus, double overhead) {
    if (groups <= cus) return 1;
    int best = 1;
    double best_cost = 1e300;
    for (int s = 1; s <= 8 && s <= iters; ++s) {
        const double rounds = (double)((groups * s + cus - 1) / cus) / s;
        const double cost = rounds * (1.0 + overhead * s);
        if (cost < best_cost - 1e-12) { best_cost = cost; best = s; }
    }
    return best;
}

// Which fused decoder kernel a launch gets: 0 / 1 one chunk per step with dense / sparse state, 2 one 32-row tile per
// workgroup, 3 / 4 two chunks per step with dense / sparse state.
int fused_variant(int MT, long long rows_pad, int nct) {
    const int cus = cu_count();
    // few rows: one 32-row tile per workgroup, so that every tile has a CU of its own
    const bool thin = rows_pad / 32 <= cus && (*tl_opt)[CSAT_OPT_FUSED_THIN] != 1;      // (14 tiles of m and more: only when forced)
    int variant = thin ? 2 : (sparse_state((size_t)rows_pad * nct * 32 * 4) ? 1 : 0);
    // 128-row workgroups on rows of at least five chunks and three tiles of m: two chunks per step (the schedule
    // looks two steps ahead, and spreads each threshold over more than one group of MFMAs)
    // and works in whole pairs of chunks: an odd chunk count is padded with a zero chunk, not worth it for short rows
    // (image_text, 9 chunks: 0.207 ms against 0.190 ms on the one-chunk schedule)
    if (!thin && nct >= 5 && (nct % 2 == 0 || nct >= 21) && MT >= 3 && MT <= kFused2MaxMT && (*tl_opt)[CSAT_OPT_FUSED_SCHEDULE] != 1) variant += 3;
    return variant;
}

// The synthesis C = X V inside the two-chunk decoder's last iteration (csat_ista_fused2.h): bf16, d = 64, whole
// 32-row tiles per head, and V's fragments must fit the buffer of V^T they replace.
bool synthesis_in_decoder(const csat_dims& d, const Workspace& w) {
    if (!w.fused || d.dtype != CSAT_BF16 || d.d != 64 || d.n_q % 32 != 0 || (*tl_opt)[CSAT_OPT_SYNTHESIS] >= 1) return false;
    if (fused_variant(w.MT, w.rows_pad, w.nct) < 3) return false;
    return (long long)((w.nct + 1) / 2 * 2) * 32 <= w.ldn;
}

csat_status launch_ista_fused(int MT, IstaFusedArgs a, long long rows_pad, hipStream_t st) {
    const int cus = cu_count();
    const int variant = fused_variant(MT, rows_pad, a.nct);
    const bool thin = variant == 2;
    a.groups = (int)(rows_pad / (thin ? 32 : 128));
    const int nct_real = a.nct;
    if (variant >= 3) a.nct = (a.nct + 1) / 2 * 2;
    // A dense-ish iterate larger than the Infinity Cache streams through once per iteration: its accesses carry the
    // non-temporal hint on the one-chunk schedule (cross_modal: 7.97 -> 7.30 ms per launch; nothing to gain where the
    // iterate is sparse or cache-resident).  CSAT_OPT_STATE + 4 / + 8: always / never.
    {
        const int so = (*tl_opt)[CSAT_OPT_STATE];
        a.state_stream = (so & 8) ? 0 : (so & 4) ? 1 : (rows_pad * (long long)a.nct * 32 * 4 > (256ll << 20));
    }
    a.segs = fused_segments(a.groups, a.iters, cus, 20.0 / ((double)a.iters * nct_real));
    // The two-chunk kernel cuts the group-iterations of the launch into one equal share per CU instead (each group cut
    // at most once; see the kernel), unless a segment count is asked for.
    a.tape = 0;
    if (variant >= 3 && a.groups > cus) a.tape = cus;
    if (const int v = (*tl_opt)[CSAT_OPT_FUSED_SEGMENTS]; v >= 1 && v <= a.iters) { a.segs = v; a.tape = 0; }
    else if (v < 0 && variant >= 3) a.tape = -v < a.groups ? -v : a.groups;       // (tests: shares on small launches)
    if ((*tl_opt)[CSAT_OPT_FUSED_SPIN_LIMIT] != 0) a.spin_limit = (*tl_opt)[CSAT_OPT_FUSED_SPIN_LIMIT] < 0 ? 0 : (*tl_opt)[CSAT_OPT_FUSED_SPIN_LIMIT];
    // (a.sync was cleared together with the status word: run_ista)
    const long long units = a.tape > 0 ? a.tape : (long long)a.groups * a.segs;
    const unsigned grid = (unsigned)(units < cus ? units : cus);
    *tl_decoder_kernel = variant;
    switch (MT) {
#define CSAT_FUSED_CASE(N) case N: HIP_TRY(ista_fused_launch_mt##N(variant, a, grid, st)); return CSAT_OK;
        CSAT_FUSED_CASE(1) CSAT_FUSED_CASE(2) CSAT_FUSED_CASE(3) CSAT_FUSED_CASE(4)
        CSAT_FUSED_CASE(5) CSAT_FUSED_CASE(6) CSAT_FUSED_CASE(7) CSAT_FUSED_CASE(8)
        CSAT_FUSED_CASE(9) CSAT_FUSED_CASE(10) CSAT_FUSED_CASE(11) CSAT_FUSED_CASE(12)
        CSAT_FUSED_CASE(13) CSAT_FUSED_CASE(14) CSAT_FUSED_CASE(15) CSAT_FUSED_CASE(16)
#undef CSAT_FUSED_CASE
    }
    return CSAT_ERR_SHAPE;
}

// ISTA on rows of Y (float, leading dimension ldY).  Generic decoder: w.R must already hold Y in
// operand layout (the first residual, since x^0 = 0); the final state is left in w.Xs (float mode)
// or w.Xb (bf16 mode).  Fused decoder (bf16, m <= 512): Y must be w.A-style rows with
// ldY == w.ldy and zero pads; the final iterate is left in w.Xb.
template <typename T>
csat_status run_ista(const csat_dims& d, const Workspace& w, const float* Y, long long ldY, float lambda, float mu,
                     int iters, float* Xout, hipStream_t st, const T* Vsyn = nullptr, T* Csyn = nullptr, bool y_tiled = false) {
    constexpr bool kBf16 = sizeof(T) == 2;
    const long long rows = (long long)d.B * d.H * d.n_q;
    const float theta = mu * lambda;
    // word 0 of the status block: set by the fused decoder when its bounded wait gives up
    // (and, in the same launch, the fused decoder's unit counter and progress words: 2 + one per group of 32 rows at most)
    const long long sync_words = w.fused ? 2 + w.rows_pad / 32 : 0;
    hipLaunchKernelGGL(set_word_kernel, dim3((unsigned)(sync_words > 256 ? (sync_words + 255) / 256 : 1)), dim3(256), 0, st, w.Status,
                       (w.fused && (*tl_opt)[CSAT_OPT_INJECT_DECODER_ERROR]) ? 1 : 0, (uint32_t*)w.FusedSync, sync_words);
    HIP_TRY(hipGetLastError());
    *tl_decoder_kernel = -1;
    if (w.fused) {
        IstaFusedArgs a{w.PhiPack, Y, w.Xs, w.Mask, w.Xb, Xout, rows, d.n, w.nct, (int)ldY, (int)w.ldn, iters, mu, theta,
                        0, 1, w.FusedSync, w.Hand, w.Status, kFusedSpinLimit};
        // Vsyn (the caller checked synthesis_in_decoder): C = X V in the kernel's last iteration, from V's fragments in
        // the buffer of V^T; no bf16 copy of the iterate then
        a.y_tiled = y_tiled ? 1 : 0;
        const bool syn = Vsyn && Csyn;
        if (syn) {
            Timed tm(w, CSAT_K_LAYOUT, st);
            const int nct2 = (w.nct + 1) / 2 * 2;
            const long long total = (long long)d.B * d.H * nct2 * 256;
            hipLaunchKernelGGL(pack_v_fragments_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                               (const bf16_t*)Vsyn, d.n, nct2, total, (uint4*)w.VT);
            HIP_TRY(hipGetLastError());
            a.Xb = nullptr;
            a.Vf = (const uint4*)w.VT; a.C = (bf16_t*)Csyn; a.n_q = d.n_q;
        }
        // the kernel writes the bf16 copy in whole 32-column chunks; operand rows are padded further
        // (the GEMM reads them; the synthesis straight from V stops at column n)
        if (!syn && !synthesis_is_direct<T>(d) && w.ldn > (long long)w.nct * 32) CSAT_TRY(fill_zero(w.Xb, (size_t)rows * w.ldn * 2, st));
        {
            Timed tm(w, CSAT_K_UPDATE, st);
            CSAT_TRY(launch_ista_fused(w.MT, a, w.rows_pad, st));
        }
        // a decoder that gave up leaves part of the iterate unwritten: make that visible in the outputs
        // (NaN in X and, through the synthesis product, in C) as well as in csat_decoder_status
        hipLaunchKernelGGL(poison_on_error_kernel, dim3(256), dim3(256), 0, st, w.Status, (uint32_t*)Xout,
                           Xout ? rows * (long long)d.n : 0ll, syn ? (uint32_t*)Csyn : (uint32_t*)w.Xb,
                           syn ? rows * (long long)d.d / 2 : rows * w.ldn / 2);
        HIP_TRY(hipGetLastError());
        return CSAT_OK;
    }
    for (int t = 0; t < iters; ++t) {
        if (t > 0) {   // residual r = y - Phi x
            GemmArgs g{kBf16 ? (const void*)w.Xb : (const void*)w.Xs, w.ldn, 0, w.PhiP, w.ldn, 0, 0, d.m, d.n, 0};
            g.M = (int)rows;
            Timed tm(w, CSAT_K_RESIDUAL, st);
            if (w.split > 1 && use_big_gemm<T>(g, w.ldm)) {     // partial products along K, then r = y - their sum
                GemmArgs gs = g;
                gs.K = (int)(w.ldn / w.split);
                gs.strideA = gs.strideB = gs.K;
                EpiStore<float> ep{w.SplitP, w.ldm, rows * w.ldm, nullptr, 0, 0, 1.f, (int)rows, d.m};
                CSAT_TRY(launch_gemm_big(gs, w.ldm, w.split, ep, st));
                const long long total = rows * w.ldm;
                hipLaunchKernelGGL(residual_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, Y, ldY,
                                   w.SplitP, w.split, rows * w.ldm, (bf16_t*)w.R, w.ldm, rows, d.m);
                HIP_TRY(hipGetLastError());
            } else if (use_big_gemm<T>(g, w.ldm) && ldY % 4 == 0 && aligned16(Y)) {
                EpiResidualTiled er{Y, ldY, (bf16_t*)w.R, w.ldm, rows, d.m};
                g.K = (int)round_up(g.K, 64);
                CSAT_TRY(launch_gemm_big(g, w.ldm, 1, er, st));
            } else {
                EpiResidual<T> er{Y, ldY, (T*)w.R, w.ldm, rows, d.m};
                CSAT_TRY((gemm<T>(g, w.ldm, 1, er, st)));
            }
        }
        GemmArgs g{w.R, w.ldm, 0, w.PhiT, w.ldm, 0, (int)rows, d.n, d.m, 0};
        Timed tm(w, CSAT_K_UPDATE, st);
        if (use_big_gemm<T>(g, w.ldn)) {   // large-tile kernel: state in accumulator order
            EpiIstaUpdateTiled eu{(f32x4*)w.Xs, w.ldn / 32, w.Mask, w.Xb, w.ldn, (t == iters - 1) ? Xout : nullptr,
                                  mu, theta, rows, d.n, t == 0};
            g.K = (int)round_up(g.K, 64);
            CSAT_TRY(launch_gemm_big(g, w.ldn, 1, eu, st));
            continue;
        }
        EpiIstaUpdate eu{w.Xs, kBf16 ? w.Xb : nullptr, w.ldn, (t == iters - 1) ? Xout : nullptr,
                         mu, theta, rows, d.n, t == 0};
        CSAT_TRY((gemm<T>(g, w.ldn, 1, eu, st)));
    }
    return CSAT_OK;
}

// C = X V per head from the decoder state; V: as the caller holds it, or nullptr when only w.VT (its transpose) is there
template <typename T>
csat_status run_synthesis(const csat_dims& d, const Workspace& w, T* C, hipStream_t st, const T* V = nullptr) {
    constexpr bool kBf16 = sizeof(T) == 2;
    const int BH = d.B * d.H;
    if constexpr (kBf16) {
        if (V && synthesis_is_direct<T>(d)) {
            MeasureDirectArgs a{};
            a.Phi = w.Xb; a.ldp = w.ldn; a.strideA = (long long)d.n_q * w.ldn;
            a.ncols = (int)round_up(d.n, 8);         // (the operand's columns from n on are zero)
            a.K = (const bf16_t*)V; a.V = nullptr; a.strideX = (long long)d.n * d.d;
            a.m = d.n_q; a.n = d.n; a.MT = (d.n_q + 31) / 32;
            a.Kc = (bf16_t*)C;
            a.heads = BH;
            a.blocks_per_head = (a.MT + 3) / 4;
            const dim3 grid((unsigned)(8 * ((BH + 7) / 8) * a.blocks_per_head));
            Timed tm(w, CSAT_K_SYNTHESIS, st);
            const bool deep = d.n >= 4096;
            if (d.d == 64) {
                if (deep) hipLaunchKernelGGL((measure_direct_kernel<2, 64, 4, false>), grid, dim3(256), 0, st, a);
                else hipLaunchKernelGGL((measure_direct_kernel<2, 64, 2, false>), grid, dim3(256), 0, st, a);
            } else {
                if (deep) hipLaunchKernelGGL((measure_direct_kernel<4, 64, 4, false>), grid, dim3(256), 0, st, a);
                else hipLaunchKernelGGL((measure_direct_kernel<4, 64, 2, false>), grid, dim3(256), 0, st, a);
            }
            HIP_TRY(hipGetLastError());
            return CSAT_OK;
        }
    }
    GemmArgs g{kBf16 ? (const void*)w.Xb : (const void*)w.Xs, w.ldn, (long long)d.n_q * w.ldn,
               w.VT, w.ldn, (long long)d.d * w.ldn, d.n_q, d.d, d.n, 0};
    EpiStore<T> ec{C, d.d, (long long)d.n_q * d.d, nullptr, 0, 0, 1.f, d.n_q, d.d};
    Timed tm(w, CSAT_K_SYNTHESIS, st);
    return gemm<T>(g, d.d, BH, ec, st);
}

template <typename T>
csat_status measure_t(const csat_dims& d, const Workspace& w, const void* PhiK, const void* Phi, const void* K,
                      const void* V, void* Kc, void* Vc, hipStream_t st) {
    const bool separate = PhiK && PhiK != Phi;
    CSAT_TRY(prepare_phi<T>(d, w, (const T*)Phi, !measure_reads_raw_phi<T>(d, separate), false, st));
    return run_measure<T>(d, w, (const T*)K, (const T*)V, (T*)Kc, (T*)Vc, nullptr, measure_is_direct<T>(d, separate), false, st, (const T*)PhiK,
                          (const T*)Phi);
}

template <typename T>
csat_status attention_t(const csat_dims& d, const Workspace& w, const void* Q, const void* Kc, const void* Vc,
                        float* A, void* Z, hipStream_t st) {
    const int BH = d.B * d.H;
    {
        Timed tm(w, CSAT_K_LAYOUT, st);
        CSAT_TRY(transpose_pack<T>((const T*)Vc, (T*)w.VcT, w.ldm, BH, d.m, d.d, st));
    }
    return run_attention<T>(d, w, (const T*)Q, (const T*)Kc, (const T*)w.VcT, A ? A : w.A, A ? (long long)d.m : w.ldy, (T*)w.R, (T*)Z, false, st);
}

template <typename T>
csat_status recover_t(const csat_dims& d, const Workspace& w, const float* Y, const void* Phi, float lambda,
                      float mu, int iters, float* X, const void* V, void* C, hipStream_t st) {
    const int BH = d.B * d.H;
    const long long rows = (long long)BH * d.n_q;
    const bool want_c = V && C;
    if (iters == 0) {
        if (X) CSAT_TRY(fill_zero(X, (size_t)rows * d.n * 4, st));
        if (want_c) CSAT_TRY(fill_zero(C, (size_t)rows * d.d * sizeof(T), st));
        return CSAT_OK;
    }
    CSAT_TRY(prepare_phi<T>(d, w, (const T*)Phi, false, true, st));
    {
        Timed tm(w, CSAT_K_LAYOUT, st);
        if (w.fused) CSAT_TRY((pack_rows<float, float>(Y, d.m, w.A, w.ldy, rows, d.m, st)));
        else CSAT_TRY((pack_rows<float, T>(Y, d.m, (T*)w.R, w.ldm, rows, d.m, st)));
        if (want_c && !synthesis_is_direct<T>(d)) CSAT_TRY(transpose_pack<T>((const T*)V, (T*)w.VT, w.ldn, BH, d.n, d.d, st));
    }
    CSAT_TRY(run_ista<T>(d, w, w.fused ? w.A : Y, w.fused ? w.ldy : (long long)d.m, lambda, mu, iters, X, st));
    if (want_c) CSAT_TRY(run_synthesis<T>(d, w, (T*)C, st, (const T*)V));
    return CSAT_OK;
}

template <typename T>
csat_status forward_t(const csat_dims& d, const Workspace& w, const void* Q, const void* K, const void* V,
                      const void* PhiK, const void* Phi, float lambda, float mu, int iters, void* C, void* Z,
                      float* X, hipStream_t st) {
    const bool separate = PhiK && PhiK != Phi;
    CSAT_TRY(prepare_phi<T>(d, w, (const T*)Phi, !measure_reads_raw_phi<T>(d, separate), iters > 0, st));
    const bool need_z = Z || iters == 0;
    T* zdst = (iters == 0) ? (T*)C : (T*)Z;
    bool kc_packed = false, v_packed = false;
    // (then nothing reads V^T: the one-kernel measurement takes V as it is)
    const bool syn = iters > 0 && synthesis_in_decoder(d, w) && measure_is_direct<T>(d, separate);
    CSAT_TRY(run_measure<T>(d, w, (const T*)K, (const T*)V, (T*)w.Kc, (T*)w.Vc, need_z ? (T*)w.VcT : nullptr, syn || synthesis_is_direct<T>(d), true, st,
                            (const T*)PhiK, (const T*)Phi, need_z, &kc_packed,
                            // (the two-sweep form of the kernel leaves Z to a product GEMM: with the product's registers
                            // on top it spills; long_video 4.0 ms against 1.2)
                            attention_is_fused<T>(d, w, true) && attention_packed_v_fits(w.MT, d.d) ? &v_packed : nullptr));
    // the operand copy of A~ feeds the Z product as a GEMM and the GEMM-pair decoder; the fused decoder reads A~ itself
    T* pcopy = ((need_z && !v_packed) || !w.fused) ? (T*)w.R : nullptr;
    // A~ in accumulator tiles between the attention kernel and the two-chunk decoder: both then move whole 1 KB pieces
    // per instruction instead of 16-byte pieces of 32 rows.  Needs whole 32-row tiles per head and the forms of the two
    // kernels that support it (single sweep with the scores kept in the accumulator file; the two-chunk decoder).
    bool y_tiled = false;
    if constexpr (sizeof(T) == 2) {
        y_tiled = iters > 0 && w.fused && d.n_q % 32 == 0 && (*tl_opt)[CSAT_OPT_Y_LAYOUT] != 1 &&
                  fused_variant(w.MT, w.rows_pad, w.nct) >= 3 && attention_is_fused<T>(d, w, true) &&
                  attention_single_sweep(w.MT, 2 * ((d.d + 15) / 16)) &&
                  (v_packed || (!need_z && attention_mtp(w.MT, true) == 13));
    }
    CSAT_TRY(run_attention<T>(d, w, (const T*)Q, (const T*)w.Kc, (const T*)w.VcT, w.A, w.ldy, pcopy,
                              need_z ? zdst : nullptr, true, st, nullptr, kc_packed, v_packed, y_tiled));
    if (iters == 0) {
        if (Z) HIP_TRY(hipMemcpyAsync(Z, C, (size_t)d.B * d.H * d.n_q * d.d * sizeof(T), hipMemcpyDeviceToDevice, st));
        return CSAT_OK;
    }
    if (syn) return run_ista<T>(d, w, w.A, w.ldy, lambda, mu, iters, X, st, (const T*)V, (T*)C, y_tiled);
    CSAT_TRY(run_ista<T>(d, w, w.A, w.ldy, lambda, mu, iters, X, st, nullptr, nullptr, y_tiled));
    return run_synthesis<T>(d, w, (T*)C, st, (const T*)V);
}

// Column-wise decode (n_q == n): the decoder's problems are the d feature columns of Z per head.
// Its buffers are a second carving, for the same shape with d rows per head, placed after the main
// one, followed by the transposed Z and the decoded columns.
csat_dims rd_dims(const csat_dims& d) {
    csat_dims r = d;
    r.n_q = d.d;
    return r;
}
struct RdExtra { char* ZT; float* Xout; size_t bytes; };
RdExtra carve_rd_extra(const csat_dims& d, const Workspace& wr, char* base) {
    const long long rows = (long long)d.B * d.H * d.d;
    const size_t zt = (size_t)round_up(rows * wr.ldn * 4, 256);   // a bf16 (hi | lo) pair or one float per element
    return RdExtra{base, (float*)(base + zt), zt + (size_t)round_up(rows * (long long)d.n * 4, 256)};
}

template <typename T>
csat_status forward_rd_t(const csat_dims& d, const Workspace& w, const Workspace& wr, const RdExtra& x, const void* Q,
                         const void* K, const void* V, const void* PhiK, const void* Phi, float lambda, float mu,
                         int iters, void* C, void* Z, hipStream_t st) {
    constexpr bool kBf16 = sizeof(T) == 2;
    const int BH = d.B * d.H;
    const long long rows = (long long)BH * d.d;          // decoder problems
    const csat_dims dr = rd_dims(d);
    CSAT_TRY(prepare_phi<T>(d, w, (const T*)Phi, true, false, st));
    CSAT_TRY(run_measure<T>(d, w, (const T*)K, (const T*)V, (T*)w.Kc, (T*)w.Vc, (T*)w.VcT,
                            measure_is_direct<T>(d, PhiK && PhiK != Phi), true, st, (const T*)PhiK, (const T*)Phi));
    if (iters == 0) {
        CSAT_TRY(run_attention<T>(d, w, (const T*)Q, (const T*)w.Kc, (const T*)w.VcT, w.A, w.ldy, (T*)w.R, (T*)C, true, st));
        if (Z) HIP_TRY(hipMemcpyAsync(Z, C, (size_t)BH * d.n * d.d * sizeof(T), hipMemcpyDeviceToDevice, st));
        return CSAT_OK;
    }
    const long long ldzt = kBf16 ? 2 * w.ldn : w.ldn;
    CSAT_TRY(fill_zero(x.ZT, (size_t)rows * ldzt * sizeof(T), st));
    CSAT_TRY(run_attention<T>(d, w, (const T*)Q, (const T*)w.Kc, (const T*)w.VcT, w.A, w.ldy, (T*)w.R, (T*)Z, true, st,
                              (T*)x.ZT));
    {   // Y^T [m, rows] = Phi Z^T per column, stored transposed as the decoder's measurement rows
        CSAT_TRY(fill_zero(wr.A, (size_t)rows * wr.ldy * 4, st));
        GemmArgs g{w.PhiP, w.ldn, 0, x.ZT, ldzt, 0, d.m, (int)rows, kBf16 ? (int)(2 * w.ldn) : d.n, kBf16 ? (int)(w.ldn / 8) : 0};
        EpiStore<float> ey{nullptr, 0, 0, wr.A, wr.ldy, 0, 1.f, d.m, (int)rows};
        Timed tm(w, CSAT_K_MEASURE, st);
        CSAT_TRY((gemm<T>(g, rows, 1, ey, st)));
    }
    CSAT_TRY(prepare_phi<T>(dr, wr, (const T*)Phi, false, true, st));
    if (!wr.fused) {
        Timed tm(w, CSAT_K_LAYOUT, st);
        CSAT_TRY((pack_rows<float, T>(wr.A, wr.ldy, (T*)wr.R, wr.ldm, rows, d.m, st)));
    }
    CSAT_TRY(run_ista<T>(dr, wr, wr.A, wr.ldy, lambda, mu, iters, x.Xout, st));
    {   // C[b,h,j,k] = decoded column k at token j
        Timed tm(w, CSAT_K_SYNTHESIS, st);
        dim3 grid((unsigned)((d.d + 31) / 32), (unsigned)((d.n + 31) / 32), (unsigned)BH);
        hipLaunchKernelGGL((transpose_cast_kernel<T>), grid, dim3(32, 8), 0, st, x.Xout, (T*)C, d.d, d.n);
        HIP_TRY(hipGetLastError());
    }
    return CSAT_OK;
}

// Buffers of the unrolled (LISTA) decoder, carved after the main workspace.
struct ListaExtra {
    char* D;        // [n, ldn]     S - I, operand layout
    float* W;       // [rows_pad, ldn]  B y (row-major, or in accumulator order on the large-tile path)
    float* StateF;  // [rows_pad, ldn]  fp32 iterate (bf16 mode; in fp32 mode the operand buffers are the iterate)
    uint8_t* Mask;  // [rows_pad/32, ldn/32, 64]  non-zero float4 pieces of the iterate (large-tile path)
    char* Op[2];    // [rows, ldn]  GEMM operand of the current / next layer
    size_t bytes;
};
ListaExtra carve_lista(const csat_dims& d, const Workspace& w, char* base) {
    const long long rows = (long long)d.B * d.H * d.n_q;
    const size_t e = esize(d.dtype);
    ListaExtra x{};
    size_t off = 0;
    auto take = [&](size_t nbytes) {
        char* p = base + off;
        off += (size_t)round_up((long long)nbytes, 256);
        return p;
    };
    x.D = take((size_t)d.n * w.ldn * e);
    x.W = (float*)take((size_t)w.rows_pad * w.ldn * 4);
    x.StateF = (float*)take(d.dtype == CSAT_BF16 ? (size_t)w.rows_pad * w.ldn * 4 : 0);
    x.Mask = (uint8_t*)take(d.dtype == CSAT_BF16 ? (size_t)(w.rows_pad / 32) * (w.ldn / 32) * 64 : 0);
    x.Op[0] = take((size_t)rows * w.ldn * e);
    x.Op[1] = take((size_t)rows * w.ldn * e);
    x.bytes = off;
    return x;
}

template <typename T>
csat_status lista_t(const csat_dims& d, const Workspace& w, const ListaExtra& x, const float* Y, const void* S,
                    const void* Bw, const float* thetas, int iters, float* X, const void* V, void* C, hipStream_t st) {
    constexpr bool kBf16 = sizeof(T) == 2;
    const int BH = d.B * d.H;
    const long long rows = (long long)BH * d.n_q;
    const bool want_c = V && C;
    if (iters == 0) {
        if (X) CSAT_TRY(fill_zero(X, (size_t)rows * d.n * 4, st));
        if (want_c) CSAT_TRY(fill_zero(C, (size_t)rows * d.d * sizeof(T), st));
        return CSAT_OK;
    }
    // bf16 problems large enough for the 256-wide kernel take tile-level epilogues
    const bool tiled = kBf16 && use_big_gemm<T>(GemmArgs{nullptr, w.ldn, 0, nullptr, w.ldn, 0, (int)rows, d.n, d.n, 0}, w.ldn) &&
                       use_big_gemm<T>(GemmArgs{nullptr, w.ldm, 0, nullptr, w.ldm, 0, (int)rows, d.n, d.m, 0}, w.ldn) &&
                       lista_choice() != 1;
    {
        Timed tm(w, CSAT_K_LAYOUT, st);
        CSAT_TRY((pack_rows<T, T>((const T*)Bw, d.m, (T*)w.PhiT, w.ldm, d.n, d.m, st)));
        const long long total = (long long)d.n * w.ldn;
        hipLaunchKernelGGL((sub_identity_pack_kernel<T>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           (const T*)S, d.n, (T*)x.D, w.ldn);
        HIP_TRY(hipGetLastError());
        CSAT_TRY((pack_rows<float, T>(Y, d.m, (T*)w.R, w.ldm, rows, d.m, st)));
        if (want_c && !synthesis_is_direct<T>(d)) CSAT_TRY(transpose_pack<T>((const T*)V, (T*)w.VT, w.ldn, BH, d.n, d.d, st));
        // alpha^(0) = 0
        CSAT_TRY(fill_zero(x.Op[0], (size_t)rows * w.ldn * sizeof(T), st));
        if (kBf16 && !tiled) CSAT_TRY(fill_zero(x.StateF, (size_t)rows * w.ldn * 4, st));
    }
    {   // W = B y for every row
        GemmArgs g{w.R, w.ldm, 0, w.PhiT, w.ldm, 0, (int)rows, d.n, d.m, 0};
        Timed tm(w, CSAT_K_RESIDUAL, st);
        if (tiled) {
            EpiStoreAccTiled ew{(f32x4*)x.W, w.ldn / 32, w.ldn, rows};
            g.K = (int)round_up(g.K, 64);
            CSAT_TRY(launch_gemm_big(g, w.ldn, 1, ew, st));
        } else {
            EpiStore<float> ew{x.W, w.ldn, 0, nullptr, 0, 0, 1.f, (int)rows, d.n};
            CSAT_TRY((gemm<T>(g, d.n, 1, ew, st)));
        }
    }
    for (int t = 0; t < iters; ++t) {
        char* cur = x.Op[t & 1];
        char* nxt = x.Op[(t + 1) & 1];
        GemmArgs g{cur, w.ldn, 0, x.D, w.ldn, 0, (int)rows, d.n, d.n, 0};
        if (tiled) {    // accumulators start from W; the iterate is kept like the ISTA decoder's (sparse, accumulator order)
            EpiListaUpdateTiled eu{{(f32x4*)x.StateF, w.ldn / 32, x.Mask, (bf16_t*)nxt, w.ldn,
                                    (t == iters - 1) ? X : nullptr, 1.f, thetas[t], rows, d.n, t == 0},
                                   (const f32x4*)x.W};
            g.K = t == 0 ? 64 : (int)round_up(g.K, 64);      // alpha^(0) = 0: one K step over the zero operand
            Timed tm(w, CSAT_K_UPDATE, st);
            CSAT_TRY(launch_gemm_big(g, w.ldn, 1, eu, st));
            continue;
        }
        EpiListaUpdate eu{kBf16 ? x.StateF : (const float*)cur, kBf16 ? x.StateF : (float*)nxt, w.ldn, x.W,
                          kBf16 ? (bf16_t*)nxt : nullptr, (t == iters - 1) ? X : nullptr, thetas[t], rows, d.n};
        Timed tm(w, CSAT_K_UPDATE, st);
        CSAT_TRY((gemm<T>(g, w.ldn, 1, eu, st)));
    }
    if (want_c) {
        Workspace wf = w;          // the synthesis reads the final operand buffer
        if (kBf16) wf.Xb = (bf16_t*)x.Op[iters & 1];
        else wf.Xs = (float*)x.Op[iters & 1];
        CSAT_TRY(run_synthesis<T>(d, wf, (T*)C, st, (const T*)V));
    }
    return CSAT_OK;
}

// Buffers of the matching-pursuit decoder, carved after the main workspace.
struct OmpExtra {
    float* Cm;     // [rows, ldn]    correlations of the current residuals with every column
    float* Rf;     // [rows, mq]     fp32 residuals
    float* Qb;     // [rows, k, mq]  orthonormalised picked columns
    float* Tri;    // [rows, k, k]   triangular factor
    float* Z;      // [rows, k]      Q^T y
    int* picks;    // [rows, k]
    int mq;
    size_t bytes;
};
OmpExtra carve_omp(const csat_dims& d, const Workspace& w, int k, char* base) {
    const long long rows = (long long)d.B * d.H * d.n_q;
    OmpExtra x{};
    x.mq = (int)round_up(d.m, 64);
    size_t off = 0;
    auto take = [&](size_t nbytes) {
        char* p = base + off;
        off += (size_t)round_up((long long)nbytes, 256);
        return p;
    };
    x.Cm = (float*)take((size_t)rows * w.ldn * 4);
    x.Rf = (float*)take((size_t)rows * x.mq * 4);
    x.Qb = (float*)take((size_t)rows * k * x.mq * 4);
    x.Tri = (float*)take((size_t)rows * k * k * 4);
    x.Z = (float*)take((size_t)rows * k * 4);
    x.picks = (int*)take((size_t)rows * k * 4);
    x.bytes = off;
    return x;
}

template <typename T>
csat_status omp_t(const csat_dims& d, const Workspace& w, const OmpExtra& x, const float* Y, const void* Phi, int k,
                  float* X, int* picks, const void* V, void* C, hipStream_t st) {
    const int BH = d.B * d.H;
    const long long rows = (long long)BH * d.n_q;
    const bool want_c = V && C;
    if (X) CSAT_TRY(fill_zero(X, (size_t)rows * d.n * 4, st));
    if (k == 0) {
        if (want_c) CSAT_TRY(fill_zero(C, (size_t)rows * d.d * sizeof(T), st));
        return CSAT_OK;
    }
    const unsigned row_blocks = (unsigned)((rows + 3) / 4);
    {
        Timed tm(w, CSAT_K_LAYOUT, st);
        CSAT_TRY(transpose_pack<T>((const T*)Phi, (T*)w.PhiT, w.ldm, 1, d.m, d.n, st));
        CSAT_TRY((pack_rows<float, T>(Y, d.m, (T*)w.R, w.ldm, rows, d.m, st)));        // r = y
        CSAT_TRY((pack_rows<float, float>(Y, d.m, x.Rf, x.mq, rows, d.m, st)));
    }
    for (int it = 0; it < k; ++it) {
        {   // correlations of every residual with every column
            GemmArgs g{w.R, w.ldm, 0, w.PhiT, w.ldm, 0, (int)rows, d.n, d.m, 0};
            EpiStoreStream ec{x.Cm, w.ldn, (int)rows, d.n};
            Timed tm(w, CSAT_K_UPDATE, st);
            CSAT_TRY((gemm<T>(g, d.n, 1, ec, st)));
        }
        Timed tm(w, CSAT_K_RESIDUAL, st);
        hipLaunchKernelGGL(omp_pick_kernel, dim3(row_blocks), dim3(256), 0, st, x.Cm, w.ldn, rows, d.n, x.picks, k, it);
#define CSAT_OMP_UPDATE(MQ_)                                                                                              \
    hipLaunchKernelGGL((omp_update_kernel<T, MQ_>), dim3(row_blocks), dim3(256), 0, st, (const T*)w.PhiT, w.ldm, d.m, x.picks, \
                       k, it, x.Qb, x.Tri, x.Z, x.Rf, x.mq, (T*)w.R, w.ldm, rows)
        if (x.mq <= 256) CSAT_OMP_UPDATE(4);
        else if (x.mq <= 512) CSAT_OMP_UPDATE(8);
        else CSAT_OMP_UPDATE(16);
#undef CSAT_OMP_UPDATE
        HIP_TRY(hipGetLastError());
    }
    Timed tm(w, CSAT_K_SYNTHESIS, st);
    hipLaunchKernelGGL((omp_finish_kernel<T>), dim3(row_blocks), dim3(256), 0, st, x.Tri, x.Z, x.picks, k, rows, d.n_q, d.n, d.d,
                       X, picks, want_c ? (const T*)V : nullptr, want_c ? (T*)C : nullptr);
    HIP_TRY(hipGetLastError());
    return CSAT_OK;
}

template <typename T>
csat_status hadamard_t(const csat_dims& d, const Workspace& w, const float* Y, long long ldY, const int* rows_of_h,
                       const signed char* signs, float lambda, float mu, int iters, float* X, const void* V, void* C,
                       hipStream_t st) {
    constexpr bool kBf16 = sizeof(T) == 2;
    const int BH = d.B * d.H;
    const long long rows = (long long)BH * d.n_q;
    const bool want_c = V && C;
    if (iters == 0) {
        if (X) CSAT_TRY(fill_zero(X, (size_t)rows * d.n * 4, st));
        if (want_c) CSAT_TRY(fill_zero(C, (size_t)rows * d.d * sizeof(T), st));
        return CSAT_OK;
    }
    int N = 1, logN = 0;
    while (N < d.n) { N *= 2; ++logN; }
    float scale = 1.f / sqrtf((float)d.m);
    if (kBf16) scale = bf2f_host(f2bf_host(scale));       // the explicit matrix would hold this value
    HadamardArgs a{Y, ldY, rows_of_h, signs, X, want_c ? (kBf16 ? (void*)w.Xb : (void*)w.Xs) : nullptr, w.ldn, rows,
                   d.n, d.m, N, logN, iters, mu, mu * lambda, scale};
    const bool in_regs = N >= 512 && hadamard_choice() != 1;      // the iterate in registers (two values per thread at least)
    const size_t lds_bytes = ista_hadamard_lds_bytes(N, d.m), reg_lds = (size_t)(fwht_pad(N) + 1 + 2 * d.m) * 4;
    if ((in_regs ? reg_lds : lds_bytes) > kLdsPerWorkgroup) return CSAT_ERR_SHAPE;     // the row's buffers must fit LDS
    {
        Timed tm(w, CSAT_K_LAYOUT, st);
        if (want_c && !synthesis_is_direct<T>(d)) CSAT_TRY(transpose_pack<T>((const T*)V, (T*)w.VT, w.ldn, BH, d.n, d.d, st));
    }
    {
        Timed tm(w, CSAT_K_UPDATE, st);
        const long long cap = (long long)cu_count() * 16;
        const dim3 grid((unsigned)(rows < cap ? rows : cap));
#define CSAT_HADAMARD_LAUNCH(NT_)                                                                                     \
    do {                                                                                                              \
        HIP_TRY(hipFuncSetAttribute((const void*)ista_hadamard_kernel<T, NT_>, hipFuncAttributeMaxDynamicSharedMemorySize, \
                                    (int)lds_bytes));                                                                 \
        hipLaunchKernelGGL((ista_hadamard_kernel<T, NT_>), grid, dim3(NT_), lds_bytes, st, a);                         \
    } while (0)
#define CSAT_HADAMARD_REG_LAUNCH(NT_, VPT_)                                                                              \
    do {                                                                                                              \
        HIP_TRY(hipFuncSetAttribute((const void*)ista_hadamard_reg_kernel<T, NT_, VPT_>,                              \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)reg_lds));                       \
        hipLaunchKernelGGL((ista_hadamard_reg_kernel<T, NT_, VPT_>), grid, dim3(NT_), reg_lds, st, a, inv);           \
    } while (0)
        if (in_regs) {
            int* inv = (int*)w.PhiT;                   // N ints; the stored-matrix operands are not used on this path
            hipLaunchKernelGGL(hadamard_inverse_fill_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, st, inv, N);
            hipLaunchKernelGGL(hadamard_inverse_scatter_kernel, dim3((unsigned)((d.m + 255) / 256)), dim3(256), 0, st,
                               rows_of_h, d.m, N, inv);
            // threads per row: N/16 where that is a whole wavefront, so that a pass can take four butterfly
            // stages (16 values per thread) and a transform needs about log2 N / 4 barriers
            if (N == 512) CSAT_HADAMARD_REG_LAUNCH(64, 8);
            else if (N == 1024) CSAT_HADAMARD_REG_LAUNCH(64, 16);
            else if (N == 2048) CSAT_HADAMARD_REG_LAUNCH(128, 16);
            else if (N == 4096) CSAT_HADAMARD_REG_LAUNCH(256, 16);
            else if (N == 8192) CSAT_HADAMARD_REG_LAUNCH(512, 16);
            else CSAT_HADAMARD_REG_LAUNCH(512, 32);
        }
        else if (N <= 2048) CSAT_HADAMARD_LAUNCH(256);
        else if (N <= 4096) CSAT_HADAMARD_LAUNCH(512);
        else CSAT_HADAMARD_LAUNCH(1024);
#undef CSAT_HADAMARD_REG_LAUNCH
#undef CSAT_HADAMARD_LAUNCH
        HIP_TRY(hipGetLastError());
    }
    if (want_c) CSAT_TRY(run_synthesis<T>(d, w, (T*)C, st, (const T*)V));
    return CSAT_OK;
}

// K~ and V~ by transforms (no stored Phi)
template <typename T>
csat_status measure_hadamard_t(const csat_dims& d, const int* rows_of_h, const signed char* signs, const void* K,
                               const void* V, void* Kc, void* Vc, Profiler* prof, hipStream_t st, bf16_t* KcHL = nullptr) {
    constexpr bool kBf16 = sizeof(T) == 2;
    constexpr int CB = 16 / (int)sizeof(T);
    const int BH = d.B * d.H;
    int N = 1, logN = 0;
    while (N < d.n) { N *= 2; ++logN; }
    float scale = 1.f / sqrtf((float)d.m);
    if (kBf16) scale = bf2f_host(f2bf_host(scale));       // the explicit matrix would hold this value
    const size_t col_bytes = (size_t)(fwht_pad(N) + 1) * 4;
    int held = (int)((kLdsPerWorkgroup - 8192) / col_bytes);
    if (held < 1 || BH > 65535) return CSAT_ERR_SHAPE;
    held = held > CB ? CB : held;
    const size_t lds_bytes = held * col_bytes;
    const dim3 grid((unsigned)((d.d + CB - 1) / CB), (unsigned)BH);
    Workspace w{};
    w.prof = prof;
    Timed tm(w, CSAT_K_MEASURE, st);
#define CSAT_MEASURE_HADAMARD(NT_)                                                                                      \
    do {                                                                                                              \
        HIP_TRY(hipFuncSetAttribute((const void*)measure_hadamard_kernel<T, NT_>,                                     \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));                     \
        hipLaunchKernelGGL((measure_hadamard_kernel<T, NT_>), grid, dim3(NT_), lds_bytes, st, (const T*)K, (T*)Kc,    \
                           rows_of_h, signs, d.n, d.d, d.m, N, logN, scale, held, KcHL);                              \
        hipLaunchKernelGGL((measure_hadamard_kernel<T, NT_>), grid, dim3(NT_), lds_bytes, st, (const T*)V, (T*)Vc,    \
                           rows_of_h, signs, d.n, d.d, d.m, N, logN, scale, held, (bf16_t*)nullptr);                  \
    } while (0)
    if (N <= 2048) CSAT_MEASURE_HADAMARD(256);
    else if (N <= 4096) CSAT_MEASURE_HADAMARD(512);
    else CSAT_MEASURE_HADAMARD(1024);
#undef CSAT_MEASURE_HADAMARD
    HIP_TRY(hipGetLastError());
    return CSAT_OK;
}

// The whole block with the structured matrix: measurement and decoder by transforms, no stored Phi.
template <typename T>
csat_status forward_hadamard_t(const csat_dims& d, const Workspace& w, const void* Q, const void* K, const void* V,
                               const int* rows_of_h, const signed char* signs, float lambda, float mu, int iters, void* C,
                               void* Z, float* X, hipStream_t st) {
    constexpr bool kBf16 = sizeof(T) == 2;
    const int BH = d.B * d.H;
    CSAT_TRY(measure_hadamard_t<T>(d, rows_of_h, signs, K, V, w.Kc, w.Vc, w.prof, st, kBf16 ? w.KcHL : nullptr));
    const bool need_z = Z || iters == 0;
    T* zdst = (iters == 0) ? (T*)C : (T*)Z;
    if (need_z) {
        Timed tm(w, CSAT_K_LAYOUT, st);
        CSAT_TRY(transpose_pack<T>((const T*)w.Vc, (T*)w.VcT, w.ldm, BH, d.m, d.d, st));
    }
    CSAT_TRY(run_attention<T>(d, w, (const T*)Q, (const T*)w.Kc, (const T*)w.VcT, w.A, w.ldy, need_z ? (T*)w.R : nullptr,
                              need_z ? zdst : nullptr, true, st));
    if (iters == 0) {
        if (Z) HIP_TRY(hipMemcpyAsync(Z, C, (size_t)BH * d.n_q * d.d * sizeof(T), hipMemcpyDeviceToDevice, st));
        return CSAT_OK;
    }
    return hadamard_t<T>(d, w, w.A, w.ldy, rows_of_h, signs, lambda, mu, iters, X, V, C, st);
}

// The column-wise reading with the structured matrix: compressed block as in forward_hadamard_t, Y = Phi Z by
// transforms on Z's feature columns, the transform-based decoder on those B*H*d problems, columns back to C.
template <typename T>
csat_status forward_rd_hadamard_t(const csat_dims& d, const Workspace& w, const Workspace& wr, const RdExtra& x,
                                  const void* Q, const void* K, const void* V, const int* rows_of_h,
                                  const signed char* signs, float lambda, float mu, int iters, void* C, void* Z,
                                  hipStream_t st) {
    constexpr bool kBf16 = sizeof(T) == 2;
    const int BH = d.B * d.H;
    const long long rows = (long long)BH * d.d;          // decoder problems
    const csat_dims dr = rd_dims(d);
    CSAT_TRY(measure_hadamard_t<T>(d, rows_of_h, signs, K, V, w.Kc, w.Vc, w.prof, st, kBf16 ? w.KcHL : nullptr));
    {
        Timed tm(w, CSAT_K_LAYOUT, st);
        CSAT_TRY(transpose_pack<T>((const T*)w.Vc, (T*)w.VcT, w.ldm, BH, d.m, d.d, st));
    }
    if (iters == 0) {
        CSAT_TRY(run_attention<T>(d, w, (const T*)Q, (const T*)w.Kc, (const T*)w.VcT, w.A, w.ldy, (T*)w.R, (T*)C, true, st));
        if (Z) HIP_TRY(hipMemcpyAsync(Z, C, (size_t)BH * d.n * d.d * sizeof(T), hipMemcpyDeviceToDevice, st));
        return CSAT_OK;
    }
    const long long ldzt = kBf16 ? 2 * w.ldn : w.ldn;
    CSAT_TRY(fill_zero(x.ZT, (size_t)rows * ldzt * sizeof(T), st));
    CSAT_TRY(run_attention<T>(d, w, (const T*)Q, (const T*)w.Kc, (const T*)w.VcT, w.A, w.ldy, (T*)w.R, (T*)Z, true, st,
                              (T*)x.ZT));
    int N = 1, logN = 0;
    while (N < d.n) { N *= 2; ++logN; }
    float scale = 1.f / sqrtf((float)d.m);
    if (kBf16) scale = bf2f_host(f2bf_host(scale));
    {
        const size_t lds_bytes = (size_t)(fwht_pad(N) + 1) * 4;
        const long long cap = (long long)cu_count() * 16;
        const dim3 grid((unsigned)(rows < cap ? rows : cap));
        Timed tm(w, CSAT_K_MEASURE, st);
#define CSAT_MEASURE_COLUMNS(NT_)                                                                                       \
    do {                                                                                                              \
        HIP_TRY(hipFuncSetAttribute((const void*)measure_columns_hadamard_kernel<T, NT_>,                             \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes));                     \
        hipLaunchKernelGGL((measure_columns_hadamard_kernel<T, NT_>), grid, dim3(NT_), lds_bytes, st, (const T*)x.ZT,  \
                           ldzt, kBf16 ? w.ldn : 0ll, rows_of_h, signs, wr.A, wr.ldy, rows, d.n, d.m, N, logN, scale);  \
    } while (0)
        if (N <= 2048) CSAT_MEASURE_COLUMNS(256);
        else if (N <= 4096) CSAT_MEASURE_COLUMNS(512);
        else CSAT_MEASURE_COLUMNS(1024);
#undef CSAT_MEASURE_COLUMNS
        HIP_TRY(hipGetLastError());
    }
    CSAT_TRY(hadamard_t<T>(dr, wr, wr.A, wr.ldy, rows_of_h, signs, lambda, mu, iters, x.Xout, nullptr, nullptr, st));
    {   // C[b,h,j,k] = decoded column k at token j
        Timed tm(w, CSAT_K_SYNTHESIS, st);
        dim3 grid((unsigned)((d.d + 31) / 32), (unsigned)((d.n + 31) / 32), (unsigned)BH);
        hipLaunchKernelGGL((transpose_cast_kernel<T>), grid, dim3(32, 8), 0, st, x.Xout, (T*)C, d.d, d.n);
        HIP_TRY(hipGetLastError());
    }
    return CSAT_OK;
}

csat_status check_ws(void* ctx, const csat_dims* dims, void* workspace, size_t workspace_bytes, Workspace* w) {
    if (!workspace) return CSAT_ERR_WORKSPACE;
    if (!aligned16(workspace)) return CSAT_ERR_ALIGN;
    *w = carve(*dims, (char*)workspace);
    w->prof = &static_cast<Context*>(ctx)->prof;
    return workspace_bytes >= w->bytes ? CSAT_OK : CSAT_ERR_WORKSPACE;
}

// The transform-based decoder keeps a row's transform buffer and measurements in LDS: checked by the entry
// points before anything is launched (hadamard_t computes the same sizes for its launch).
bool hadamard_fits_lds(int n, int m) {
    int N = 1;
    while (N < n) N *= 2;
    const bool in_regs = N >= 512 && hadamard_choice() != 1;
    const size_t need = in_regs ? (size_t)(fwht_pad(N) + 1 + 2 * m) * 4 : ista_hadamard_lds_bytes(N, m);
    return need <= kLdsPerWorkgroup;
}

// Scratch of csat_forward_static: the workspace of a small problem, held in the code object's own device memory
// so that the call allocates nothing.  Every device the library is used on holds its own copy until the process ends.
constexpr size_t kStaticScratchBytes = (size_t)48 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of this device's copy of `scratch` (looked up once per device, with that device current).
csat_status static_scratch(void** out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return CSAT_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return CSAT_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return CSAT_OK;
}

}  // namespace

extern "C" {

csat_status csat_create(void** ctx) {
    if (!ctx) return CSAT_ERR_NULL;
    Context* c = new (std::nothrow) Context{kMagic, {}};
    if (!c) return CSAT_ERR_PARAM;
    *ctx = c;
    return CSAT_OK;
}

csat_status csat_destroy(void* ctx) {
    CSAT_TRY(check_ctx(ctx));
    Context* c = static_cast<Context*>(ctx);
    c->magic = 0;
    c->prof.clear();
    delete c;
    return CSAT_OK;
}

const char* csat_status_string(csat_status s) {
    switch (s) {
        case CSAT_OK: return "ok";
        case CSAT_ERR_NULL: return "a required pointer is NULL";
        case CSAT_ERR_SHAPE: return "bad shape (non-positive dimension, m > n, d not a multiple of 8, or B*H > 65535)";
        case CSAT_ERR_DTYPE: return "unsupported dtype";
        case CSAT_ERR_ALIGN: return "pointer not 16-byte aligned";
        case CSAT_ERR_WORKSPACE: return "workspace missing or too small";
        case CSAT_ERR_PARAM: return "bad parameter (lambda < 0, step <= 0, iters < 0, or invalid context)";
        case CSAT_ERR_HIP: return "HIP runtime error";
        case CSAT_ERR_TIMEOUT: return "the decoder's bounded wait gave up; the outputs of that call are invalid";
    }
    return "unknown status";
}

csat_status csat_workspace_bytes(const csat_dims* dims, int iters, size_t* bytes) {
    CSAT_TRY(check_dims(dims));
    if (!bytes) return CSAT_ERR_NULL;
    if (iters < 0) return CSAT_ERR_PARAM;
    size_t total = carve(*dims, nullptr).bytes;
    if (dims->n_q == dims->n) {   // room for the column-wise decode as well
        const Workspace wr = carve(rd_dims(*dims), nullptr);
        total += wr.bytes + carve_rd_extra(*dims, wr, nullptr).bytes;
    }
    *bytes = total;
    return CSAT_OK;
}

// Word k of the SplitMix64 sequence started at `seed` (the state advances by a fixed odd constant, so any word
// can be formed on its own), then its output mix.
static inline uint64_t phi_word(uint64_t seed, uint64_t k) {
    uint64_t z = seed + (k + 1) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

csat_status csat_phi_fill(int kind, unsigned long long seed, int m, int n, float* phi_host) {
    if (!phi_host) return CSAT_ERR_NULL;
    if (m <= 0 || n <= 0) return CSAT_ERR_SHAPE;
    if (kind != CSAT_PHI_GAUSSIAN && kind != CSAT_PHI_RADEMACHER) return CSAT_ERR_PARAM;
    const double scale = 1.0 / std::sqrt((double)m), two_pi = 6.283185307179586476925286766559;
    const long long total = (long long)m * n;
    for (long long i = 0; i < total; ++i) {
        const uint64_t w1 = phi_word(seed, 2 * (uint64_t)i), w2 = phi_word(seed, 2 * (uint64_t)i + 1);
        double v;
        if (kind == CSAT_PHI_RADEMACHER) {
            v = (w1 >> 63) ? -1.0 : 1.0;
        } else {      // Box-Muller: u1 in (0, 1], u2 in [0, 1), 53 bits each
            const double u1 = ((double)(w1 >> 11) + 1.0) * 0x1p-53, u2 = (double)(w2 >> 11) * 0x1p-53;
            v = std::sqrt(-2.0 * std::log(u1)) * std::cos(two_pi * u2);
        }
        phi_host[i] = (float)(v * scale);
    }
    return CSAT_OK;
}

csat_status csat_phi_opnorm2(const float* phi, int m, int n, double* L) {
    if (!phi || !L) return CSAT_ERR_NULL;
    if (m <= 0 || n <= 0) return CSAT_ERR_SHAPE;
    // power iteration on G = Phi Phi^T (m x m, formed once in double; rows of G shared out over host threads,
    // every entry summed in the same order whatever the thread count)
    std::vector<double> G((size_t)m * m, 0.0);
    unsigned hw = std::thread::hardware_concurrency();
    const int nthreads = (int)std::max(1u, std::min(hw ? hw : 1u, std::min(16u, (unsigned)m)));
    auto gram_rows = [&](int t) {
        constexpr int JB = 8;                      // rows of Phi kept hot against row i
        for (int i = t; i < m; i += nthreads) {
            const float* a = phi + (size_t)i * n;
            for (int j0 = i; j0 < m; j0 += JB) {
                const int jn = std::min(JB, m - j0);
                double s[JB] = {};
                for (int k = 0; k < n; ++k) {
                    const double ak = (double)a[k];
                    for (int jj = 0; jj < jn; ++jj) s[jj] += ak * (double)phi[(size_t)(j0 + jj) * n + k];
                }
                for (int jj = 0; jj < jn; ++jj) G[(size_t)i * m + j0 + jj] = s[jj];
            }
        }
    };
    if (nthreads == 1) {
        gram_rows(0);
    } else {
        std::vector<std::thread> pool;
        for (int t = 0; t < nthreads; ++t) pool.emplace_back(gram_rows, t);
        for (auto& th : pool) th.join();
    }
    for (int i = 0; i < m; ++i)
        for (int j = i + 1; j < m; ++j) G[(size_t)j * m + i] = G[(size_t)i * m + j];
    std::vector<double> v(m), w(m);
    for (int i = 0; i < m; ++i) v[i] = 1.0 + 0.37 * std::sin(1.0 + 1.7 * i);   // generic start vector
    double lam = 0.0;
    for (int it = 0; it < 200000; ++it) {
        double nrm = 0.0;
        for (int i = 0; i < m; ++i) {
            double s = 0.0;
            const double* g = &G[(size_t)i * m];
            for (int j = 0; j < m; ++j) s += g[j] * v[j];
            w[i] = s;
            nrm += s * s;
        }
        nrm = std::sqrt(nrm);
        if (nrm == 0.0) { lam = 0.0; break; }
        double rq = 0.0, vv = 0.0;
        for (int i = 0; i < m; ++i) { rq += v[i] * w[i]; vv += v[i] * v[i]; }
        double newlam = rq / vv;
        for (int i = 0; i < m; ++i) v[i] = w[i] / nrm;
        bool done = std::fabs(newlam - lam) <= 1e-15 * std::fabs(newlam) && it > 8;
        lam = newlam;
        if (done) break;
    }
    *L = lam;
    return CSAT_OK;
}

csat_status csat_peak_copy(void* ctx, const void* src, void* dst, size_t bytes, void* stream) {
    CSAT_TRY(check_ctx(ctx));
    if (!src || !dst) return CSAT_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0) return CSAT_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(dst)) return CSAT_ERR_ALIGN;
    const long long words = (long long)(bytes / 16);
    const long long want = (words + 255) / 256;
    const unsigned grid = (unsigned)std::min<long long>(want, (long long)cu_count() * 16);
    hipLaunchKernelGGL(peak_copy_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst,
                       words);
    HIP_TRY(hipGetLastError());
    return CSAT_OK;
}

csat_status csat_peak_mfma(void* ctx, float* out, size_t out_bytes, int iters, double* flops, void* stream) {
    CSAT_TRY(check_ctx(ctx));
    if (!out || !flops) return CSAT_ERR_NULL;
    if (iters <= 0) return CSAT_ERR_PARAM;
    if (!aligned16(out)) return CSAT_ERR_ALIGN;
    const unsigned grid = (unsigned)cu_count() * 2;      // two wavefronts per SIMD
    if (out_bytes < (size_t)grid * 256 * sizeof(float)) return CSAT_ERR_WORKSPACE;
    hipLaunchKernelGGL(peak_mfma_kernel, dim3(grid), dim3(256), 0, (hipStream_t)stream, out, iters);
    HIP_TRY(hipGetLastError());
    *flops = (double)grid * 4 * (double)iters * kPeakMfmaPerIter * kPeakMfmaFlopsEach;
    return CSAT_OK;
}

csat_status csat_peak_mfma_issue(void* ctx, float* out, size_t out_bytes, int iters, int valu_per_mfma, int lds_reads_per_mfma,
                                 double* flops, void* stream) {
    CSAT_TRY(check_ctx(ctx));
    if (!out || !flops) return CSAT_ERR_NULL;
    if (iters <= 0) return CSAT_ERR_PARAM;
    if (!aligned16(out)) return CSAT_ERR_ALIGN;
    const unsigned grid = (unsigned)cu_count();          // one wavefront per SIMD
    if (out_bytes < (size_t)grid * 256 * sizeof(float)) return CSAT_ERR_WORKSPACE;
    auto launch = [&](auto kernel) -> csat_status {
        HIP_TRY(hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPeakIssueLdsBytes));
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(256), kPeakIssueLdsBytes, (hipStream_t)stream, out, iters);
        HIP_TRY(hipGetLastError());
        return CSAT_OK;
    };
    const int key = valu_per_mfma * 10 + lds_reads_per_mfma;
    switch (key) {
#define CSAT_ISSUE_CASE(KV, KL) case KV * 10 + KL: CSAT_TRY(launch(peak_issue_kernel<KV, KL>)); break;
        CSAT_ISSUE_CASE(0, 0) CSAT_ISSUE_CASE(3, 0) CSAT_ISSUE_CASE(6, 0) CSAT_ISSUE_CASE(9, 0) CSAT_ISSUE_CASE(12, 0)
        CSAT_ISSUE_CASE(0, 1) CSAT_ISSUE_CASE(3, 1) CSAT_ISSUE_CASE(6, 1) CSAT_ISSUE_CASE(0, 2)
#undef CSAT_ISSUE_CASE
        default: return CSAT_ERR_PARAM;
    }
    *flops = (double)grid * 4 * (double)iters * 8 * kPeakMfmaFlopsEach;
    return CSAT_OK;
}

csat_status csat_profile_enable(void* ctx, int on) {
    CSAT_TRY(check_ctx(ctx));
    Profiler& p = static_cast<Context*>(ctx)->prof;
    p.clear();
    p.on = on != 0;
    return CSAT_OK;
}

csat_status csat_profile_decoder_kernel(void* ctx, int* kernel) {
    CSAT_TRY(check_ctx(ctx));
    if (!kernel) return CSAT_ERR_NULL;
    *kernel = static_cast<Context*>(ctx)->decoder_kernel;
    return CSAT_OK;
}

csat_status csat_profile_read(void* ctx, int kernel_id, double* total_ms, int* launches) {
    CSAT_TRY(check_ctx(ctx));
    if (!total_ms || !launches) return CSAT_ERR_NULL;
    if (kernel_id < 0 || kernel_id >= CSAT_K_COUNT) return CSAT_ERR_PARAM;
    Profiler& p = static_cast<Context*>(ctx)->prof;
    double tot = 0.0;
    int cnt = 0;
    for (auto& s : p.spans) {
        if (s.kid != kernel_id) continue;
        float ms = 0.f;
        HIP_TRY(hipEventSynchronize(s.b));
        HIP_TRY(hipEventElapsedTime(&ms, s.a, s.b));
        tot += ms;
        ++cnt;
    }
    *total_ms = tot;
    *launches = cnt;
    return CSAT_OK;
}

#define DISPATCH(d, call_f32, call_bf16) ((d).dtype == CSAT_BF16 ? (call_bf16) : (call_f32))

csat_status csat_measure_kv(void* ctx, const csat_dims* dims, const void* PhiK, const void* PhiV, const void* K,
                            const void* V, void* Kc, void* Vc, void* workspace, size_t workspace_bytes,
                            void* stream) {
    CSAT_TRY(check_ctx(ctx));
    CSAT_TRY(check_dims(dims));
    if (!PhiK || !PhiV || !K || !V || !Kc || !Vc) return CSAT_ERR_NULL;
    if (!aligned16(PhiK) || !aligned16(PhiV) || !aligned16(K) || !aligned16(V) || !aligned16(Kc) || !aligned16(Vc))
        return CSAT_ERR_ALIGN;
    Workspace w;
    OptionScope scope(ctx);
    CSAT_TRY(check_ws(ctx, dims, workspace, workspace_bytes, &w));
    hipStream_t st = (hipStream_t)stream;
    return DISPATCH(*dims, measure_t<float>(*dims, w, PhiK, PhiV, K, V, Kc, Vc, st),
                    measure_t<bf16_t>(*dims, w, PhiK, PhiV, K, V, Kc, Vc, st));
}

csat_status csat_measure(void* ctx, const csat_dims* dims, const void* Phi, const void* K, const void* V,
                         void* Kc, void* Vc, void* workspace, size_t workspace_bytes, void* stream) {
    return csat_measure_kv(ctx, dims, Phi, Phi, K, V, Kc, Vc, workspace, workspace_bytes, stream);
}

csat_status csat_compressed_attention(void* ctx, const csat_dims* dims, const void* Q, const void* Kc,
                                      const void* Vc, float* A, void* Z, void* workspace, size_t workspace_bytes,
                                      void* stream) {
    CSAT_TRY(check_ctx(ctx));
    CSAT_TRY(check_dims(dims));
    if (!Q || !Kc || !Vc || !Z) return CSAT_ERR_NULL;
    if (!aligned16(Q) || !aligned16(Kc) || !aligned16(Vc) || !aligned16(A) || !aligned16(Z)) return CSAT_ERR_ALIGN;
    Workspace w;
    OptionScope scope(ctx);
    CSAT_TRY(check_ws(ctx, dims, workspace, workspace_bytes, &w));
    hipStream_t st = (hipStream_t)stream;
    return DISPATCH(*dims, attention_t<float>(*dims, w, Q, Kc, Vc, A, Z, st),
                    attention_t<bf16_t>(*dims, w, Q, Kc, Vc, A, Z, st));
}

csat_status csat_recover(void* ctx, const csat_dims* dims, const float* Y, const void* Phi, float lambda,
                         float step, int iters, float* X, const void* V, void* C, void* workspace,
                         size_t workspace_bytes, void* stream) {
    CSAT_TRY(check_ctx(ctx));
    CSAT_TRY(check_dims(dims));
    if (!Y || !Phi) return CSAT_ERR_NULL;
    if (!X && !(V && C)) return CSAT_ERR_NULL;
    if (!(lambda >= 0.f) || !(step > 0.f) || !std::isfinite(step) || !std::isfinite(lambda) || iters < 0)
        return CSAT_ERR_PARAM;
    if (!aligned16(Y) || !aligned16(Phi) || !aligned16(X) || !aligned16(V) || !aligned16(C)) return CSAT_ERR_ALIGN;
    Workspace w;
    OptionScope scope(ctx);
    CSAT_TRY(check_ws(ctx, dims, workspace, workspace_bytes, &w));
    hipStream_t st = (hipStream_t)stream;
    return DISPATCH(*dims, recover_t<float>(*dims, w, Y, Phi, lambda, step, iters, X, V, C, st),
                    recover_t<bf16_t>(*dims, w, Y, Phi, lambda, step, iters, X, V, C, st));
}

csat_status csat_forward(void* ctx, const csat_dims* dims, const void* Q, const void* K, const void* V,
                         const void* Phi, float lambda, float step, int iters, void* C, void* Z, float* X,
                         void* workspace, size_t workspace_bytes, void* stream) {
    return csat_forward_kv(ctx, dims, Q, K, V, Phi, Phi, lambda, step, iters, C, Z, X, workspace, workspace_bytes,
                           stream);
}

csat_status csat_forward_kv(void* ctx, const csat_dims* dims, const void* Q, const void* K, const void* V,
                            const void* PhiK, const void* Phi, float lambda, float step, int iters, void* C,
                            void* Z, float* X, void* workspace, size_t workspace_bytes, void* stream) {
    CSAT_TRY(check_ctx(ctx));
    CSAT_TRY(check_dims(dims));
    if (!Q || !K || !V || !PhiK || !Phi || !C) return CSAT_ERR_NULL;
    if (!aligned16(PhiK)) return CSAT_ERR_ALIGN;
    if (!(lambda >= 0.f) || !(step > 0.f) || !std::isfinite(step) || !std::isfinite(lambda) || iters < 0)
        return CSAT_ERR_PARAM;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(Phi) || !aligned16(C) || !aligned16(Z) ||
        !aligned16(X))
        return CSAT_ERR_ALIGN;
    Workspace w;
    OptionScope scope(ctx);
    CSAT_TRY(check_ws(ctx, dims, workspace, workspace_bytes, &w));
    hipStream_t st = (hipStream_t)stream;
    return DISPATCH(*dims, forward_t<float>(*dims, w, Q, K, V, PhiK, Phi, lambda, step, iters, C, Z, X, st),
                    forward_t<bf16_t>(*dims, w, Q, K, V, PhiK, Phi, lambda, step, iters, C, Z, X, st));
}

csat_status csat_forward_rd(void* ctx, const csat_dims* dims, const void* Q, const void* K, const void* V,
                            const void* Phi, float lambda, float step, int iters, void* C, void* Z,
                            void* workspace, size_t workspace_bytes, void* stream) {
    return csat_forward_rd_kv(ctx, dims, Q, K, V, Phi, Phi, lambda, step, iters, C, Z, workspace, workspace_bytes,
                              stream);
}

csat_status csat_forward_rd_kv(void* ctx, const csat_dims* dims, const void* Q, const void* K, const void* V,
                               const void* PhiK, const void* Phi, float lambda, float step, int iters, void* C,
                               void* Z, void* workspace, size_t workspace_bytes, void* stream) {
    CSAT_TRY(check_ctx(ctx));
    CSAT_TRY(check_dims(dims));
    if (dims->n_q != dims->n) return CSAT_ERR_SHAPE;
    if (!Q || !K || !V || !PhiK || !Phi || !C) return CSAT_ERR_NULL;
    if (!aligned16(PhiK)) return CSAT_ERR_ALIGN;
    if (!(lambda >= 0.f) || !(step > 0.f) || !std::isfinite(step) || !std::isfinite(lambda) || iters < 0)
        return CSAT_ERR_PARAM;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(Phi) || !aligned16(C) || !aligned16(Z))
        return CSAT_ERR_ALIGN;
    Workspace w;
    OptionScope scope(ctx);
    CSAT_TRY(check_ws(ctx, dims, workspace, workspace_bytes, &w));
    const csat_dims dr = rd_dims(*dims);
    Workspace wr = carve(dr, (char*)workspace + w.bytes);
    wr.prof = w.prof;
    wr.Status = w.Status;      // one status block per workspace: the column-wise decoder reports there as well
    const RdExtra x = carve_rd_extra(*dims, wr, (char*)workspace + w.bytes + wr.bytes);
    if (workspace_bytes < w.bytes + wr.bytes + x.bytes) return CSAT_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    return DISPATCH(*dims, forward_rd_t<float>(*dims, w, wr, x, Q, K, V, PhiK, Phi, lambda, step, iters, C, Z, st),
                    forward_rd_t<bf16_t>(*dims, w, wr, x, Q, K, V, PhiK, Phi, lambda, step, iters, C, Z, st));
}

csat_status csat_lista_workspace_bytes(const csat_dims* dims, int iters, size_t* bytes) {
    CSAT_TRY(check_dims(dims));
    if (!bytes) return CSAT_ERR_NULL;
    if (iters < 0) return CSAT_ERR_PARAM;
    const Workspace w = carve(*dims, nullptr);
    *bytes = w.bytes + carve_lista(*dims, w, nullptr).bytes;
    return CSAT_OK;
}

csat_status csat_recover_lista(void* ctx, const csat_dims* dims, const float* Y, const void* S, const void* Bw,
                               const float* thetas, int iters, float* X, const void* V, void* C, void* workspace,
                               size_t workspace_bytes, void* stream) {
    CSAT_TRY(check_ctx(ctx));
    CSAT_TRY(check_dims(dims));
    if (!Y || !S || !Bw) return CSAT_ERR_NULL;
    if (!X && !(V && C)) return CSAT_ERR_NULL;
    if (iters < 0 || (iters > 0 && !thetas)) return iters < 0 ? CSAT_ERR_PARAM : CSAT_ERR_NULL;
    for (int t = 0; t < iters; ++t)
        if (!(thetas[t] >= 0.f) || !std::isfinite(thetas[t])) return CSAT_ERR_PARAM;
    if (!aligned16(Y) || !aligned16(S) || !aligned16(Bw) || !aligned16(X) || !aligned16(V) || !aligned16(C))
        return CSAT_ERR_ALIGN;
    Workspace w;
    OptionScope scope(ctx);
    CSAT_TRY(check_ws(ctx, dims, workspace, workspace_bytes, &w));
    const ListaExtra x = carve_lista(*dims, w, (char*)workspace + w.bytes);
    if (workspace_bytes < w.bytes + x.bytes) return CSAT_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    return DISPATCH(*dims, lista_t<float>(*dims, w, x, Y, S, Bw, thetas, iters, X, V, C, st),
                    lista_t<bf16_t>(*dims, w, x, Y, S, Bw, thetas, iters, X, V, C, st));
}

csat_status csat_omp_workspace_bytes(const csat_dims* dims, int k, size_t* bytes) {
    CSAT_TRY(check_dims(dims));
    if (!bytes) return CSAT_ERR_NULL;
    if (k < 0 || k > kOmpMaxPicks || k > dims->m) return CSAT_ERR_PARAM;
    if (dims->m > kOmpMaxM) return CSAT_ERR_SHAPE;
    const Workspace w = carve(*dims, nullptr);
    *bytes = w.bytes + carve_omp(*dims, w, k, nullptr).bytes;
    return CSAT_OK;
}

csat_status csat_recover_omp(void* ctx, const csat_dims* dims, const float* Y, const void* Phi, int k, float* X,
                             int* picks, const void* V, void* C, void* workspace, size_t workspace_bytes,
                             void* stream) {
    CSAT_TRY(check_ctx(ctx));
    CSAT_TRY(check_dims(dims));
    if (!Y || !Phi) return CSAT_ERR_NULL;
    if (!X && !picks && !(V && C)) return CSAT_ERR_NULL;
    if (k < 0 || k > kOmpMaxPicks || k > dims->m) return CSAT_ERR_PARAM;
    if (dims->m > kOmpMaxM) return CSAT_ERR_SHAPE;
    if (!aligned16(Y) || !aligned16(Phi) || !aligned16(X) || !aligned16(picks) || !aligned16(V) || !aligned16(C))
        return CSAT_ERR_ALIGN;
    Workspace w;
    OptionScope scope(ctx);
    CSAT_TRY(check_ws(ctx, dims, workspace, workspace_bytes, &w));
    const OmpExtra x = carve_omp(*dims, w, k, (char*)workspace + w.bytes);
    if (workspace_bytes < w.bytes + x.bytes) return CSAT_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    return DISPATCH(*dims, omp_t<float>(*dims, w, x, Y, Phi, k, X, picks, V, C, st),
                    omp_t<bf16_t>(*dims, w, x, Y, Phi, k, X, picks, V, C, st));
}

csat_status csat_recover_hadamard(void* ctx, const csat_dims* dims, const float* Y, const int* rows_of_h,
                                  const signed char* signs, float lambda, float step, int iters, float* X,
                                  const void* V, void* C, void* workspace, size_t workspace_bytes, void* stream) {
    CSAT_TRY(check_ctx(ctx));
    CSAT_TRY(check_dims(dims));
    if (!Y || !rows_of_h || !signs) return CSAT_ERR_NULL;
    if (!X && !(V && C)) return CSAT_ERR_NULL;
    if (!(lambda >= 0.f) || !(step > 0.f) || !std::isfinite(step) || !std::isfinite(lambda) || iters < 0)
        return CSAT_ERR_PARAM;
    if (dims->n > kFwhtMaxN) return CSAT_ERR_SHAPE;
    if (!aligned16(Y) || !aligned16(X) || !aligned16(V) || !aligned16(C)) return CSAT_ERR_ALIGN;
    Workspace w;
    OptionScope scope(ctx);
    if (!hadamard_fits_lds(dims->n, dims->m)) return CSAT_ERR_SHAPE;
    CSAT_TRY(check_ws(ctx, dims, workspace, workspace_bytes, &w));
    hipStream_t st = (hipStream_t)stream;
    return DISPATCH(*dims, hadamard_t<float>(*dims, w, Y, dims->m, rows_of_h, signs, lambda, step, iters, X, V, C, st),
                    hadamard_t<bf16_t>(*dims, w, Y, dims->m, rows_of_h, signs, lambda, step, iters, X, V, C, st));
}

csat_status csat_forward_hadamard(void* ctx, const csat_dims* dims, const void* Q, const void* K, const void* V,
                                  const int* rows_of_h, const signed char* signs, float lambda, float step, int iters,
                                  void* C, void* Z, float* X, void* workspace, size_t workspace_bytes, void* stream) {
    CSAT_TRY(check_ctx(ctx));
    CSAT_TRY(check_dims(dims));
    if (!Q || !K || !V || !rows_of_h || !signs || !C) return CSAT_ERR_NULL;
    if (!(lambda >= 0.f) || !(step > 0.f) || !std::isfinite(step) || !std::isfinite(lambda) || iters < 0)
        return CSAT_ERR_PARAM;
    if (dims->n > kFwhtMaxN) return CSAT_ERR_SHAPE;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(C) || !aligned16(Z) || !aligned16(X))
        return CSAT_ERR_ALIGN;
    Workspace w;
    OptionScope scope(ctx);
    if (iters > 0 && !hadamard_fits_lds(dims->n, dims->m)) return CSAT_ERR_SHAPE;
    CSAT_TRY(check_ws(ctx, dims, workspace, workspace_bytes, &w));
    hipStream_t st = (hipStream_t)stream;
    return DISPATCH(*dims,
                    forward_hadamard_t<float>(*dims, w, Q, K, V, rows_of_h, signs, lambda, step, iters, C, Z, X, st),
                    forward_hadamard_t<bf16_t>(*dims, w, Q, K, V, rows_of_h, signs, lambda, step, iters, C, Z, X, st));
}

csat_status csat_forward_rd_hadamard(void* ctx, const csat_dims* dims, const void* Q, const void* K, const void* V,
                                     const int* rows_of_h, const signed char* signs, float lambda, float step,
                                     int iters, void* C, void* Z, void* workspace, size_t workspace_bytes,
                                     void* stream) {
    CSAT_TRY(check_ctx(ctx));
    CSAT_TRY(check_dims(dims));
    if (dims->n_q != dims->n || dims->n > kFwhtMaxN) return CSAT_ERR_SHAPE;
    if (!Q || !K || !V || !rows_of_h || !signs || !C) return CSAT_ERR_NULL;
    if (!(lambda >= 0.f) || !(step > 0.f) || !std::isfinite(step) || !std::isfinite(lambda) || iters < 0)
        return CSAT_ERR_PARAM;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(C) || !aligned16(Z)) return CSAT_ERR_ALIGN;
    Workspace w;
    OptionScope scope(ctx);
    CSAT_TRY(check_ws(ctx, dims, workspace, workspace_bytes, &w));
    const csat_dims dr = rd_dims(*dims);
    Workspace wr = carve(dr, (char*)workspace + w.bytes);
    wr.prof = w.prof;
    wr.Status = w.Status;
    const RdExtra x = carve_rd_extra(*dims, wr, (char*)workspace + w.bytes + wr.bytes);
    if (workspace_bytes < w.bytes + wr.bytes + x.bytes) return CSAT_ERR_WORKSPACE;
    if (iters > 0 && !hadamard_fits_lds(dims->n, dims->m)) return CSAT_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    return DISPATCH(*dims,
                    forward_rd_hadamard_t<float>(*dims, w, wr, x, Q, K, V, rows_of_h, signs, lambda, step, iters, C, Z, st),
                    forward_rd_hadamard_t<bf16_t>(*dims, w, wr, x, Q, K, V, rows_of_h, signs, lambda, step, iters, C, Z, st));
}

csat_status csat_measure_hadamard(void* ctx, const csat_dims* dims, const int* rows_of_h, const signed char* signs,
                                  const void* K, const void* V, void* Kc, void* Vc, void* stream) {
    CSAT_TRY(check_ctx(ctx));
    CSAT_TRY(check_dims(dims));
    if (!rows_of_h || !signs || !K || !V || !Kc || !Vc) return CSAT_ERR_NULL;
    if (dims->n > kFwhtMaxN) return CSAT_ERR_SHAPE;
    if (!aligned16(K) || !aligned16(V) || !aligned16(Kc) || !aligned16(Vc)) return CSAT_ERR_ALIGN;
    Profiler* prof = &static_cast<Context*>(ctx)->prof;
    hipStream_t st = (hipStream_t)stream;
    return DISPATCH(*dims, measure_hadamard_t<float>(*dims, rows_of_h, signs, K, V, Kc, Vc, prof, st),
                    measure_hadamard_t<bf16_t>(*dims, rows_of_h, signs, K, V, Kc, Vc, prof, st));
}

csat_status csat_set_option(void* ctx, int key, int value) {
    CSAT_TRY(check_ctx(ctx));
    if (key < 0 || key >= CSAT_OPT_COUNT) return CSAT_ERR_PARAM;
    static_cast<Context*>(ctx)->opt.v[key] = value;
    return CSAT_OK;
}

csat_status csat_decoder_status(void* ctx, const void* workspace, void* stream) {
    CSAT_TRY(check_ctx(ctx));
    if (!aligned16(workspace)) return CSAT_ERR_ALIGN;
    void* base = const_cast<void*>(workspace);
    if (!base) CSAT_TRY(static_scratch(&base));          // NULL: the scratch of csat_forward_static on this device
    int word = 0;
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    // the status block is the first piece of every carving, word 0 the decoder's error flag
    HIP_TRY(hipMemcpy(&word, base, sizeof(int), hipMemcpyDeviceToHost));
    return word == 0 ? CSAT_OK : CSAT_ERR_TIMEOUT;
}

csat_status csat_static_workspace_bytes(size_t* bytes) {
    if (!bytes) return CSAT_ERR_NULL;
    *bytes = kStaticScratchBytes;
    return CSAT_OK;
}

csat_status csat_forward_static(void* ctx, const csat_dims* dims, const void* Q, const void* K, const void* V,
                                const void* Phi, float lambda, float step, int iters, void* C, void* Z, float* X,
                                void* stream) {
    CSAT_TRY(check_ctx(ctx));
    CSAT_TRY(check_dims(dims));
    if (!Q || !K || !V || !Phi || !C) return CSAT_ERR_NULL;
    if (!(lambda >= 0.f) || !(step > 0.f) || !std::isfinite(step) || !std::isfinite(lambda) || iters < 0)
        return CSAT_ERR_PARAM;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(Phi) || !aligned16(C) || !aligned16(Z) ||
        !aligned16(X))
        return CSAT_ERR_ALIGN;
    OptionScope scope(ctx);
    // the row-wise block needs the main carving only
    if (carve(*dims, nullptr).bytes > kStaticScratchBytes) return CSAT_ERR_WORKSPACE;
    void* base = nullptr;
    CSAT_TRY(static_scratch(&base));
    Workspace w = carve(*dims, (char*)base);
    Profiler off;            // event creation allocates: launches of this call are never bracketed
    w.prof = &off;
    hipStream_t st = (hipStream_t)stream;
    return DISPATCH(*dims, forward_t<float>(*dims, w, Q, K, V, Phi, Phi, lambda, step, iters, C, Z, X, st),
                    forward_t<bf16_t>(*dims, w, Q, K, V, Phi, Phi, lambda, step, iters, C, Z, X, st));
}

}  // extern "C"
