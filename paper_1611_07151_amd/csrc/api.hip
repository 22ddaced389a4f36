// C boundary: argument validation, per-thread stream, algorithm choice, and the
// fire-layer and whole-network drivers that sequence the kernels.
#include "sq_internal.h"

#include <stdio.h>
#include <string.h>

#include <atomic>
#include <mutex>

namespace sq {
namespace {
thread_local hipStream_t g_stream = nullptr;
thread_local int g_last_hip = 0;
thread_local int g_dtype = SQ_F32;
// Whether a 1x1 convolution that is followed directly by global average pooling writes plane sums instead of its map
// (1), the layers run one after the other (0), or the batch size decides (-1, default: plane sums from eight images
// on; measured on whole fp32 passes, the two forms are within 3 us of each other at every batch -- at batch 1 the
// three short launches are 2.8 us faster, at batch 64 the plane sums 2.6 us -- but from there on the convolution's
// map, 676 KB per image, is neither written nor read).  Tuning hook (sq_tune_fuse_classifier).
thread_local int g_fuse_classifier = -1;
}  // namespace

hipStream_t current_stream() { return g_stream; }
int current_dtype() { return g_dtype; }

int num_cus()
{
    // filled once; two threads that race here store the same value
    static std::atomic<int> cus{0};
    int c = cus.load(std::memory_order_relaxed);
    if (!c) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            c = n;
        else
            c = 256;
        (void)hipGetLastError();
        cus.store(c, std::memory_order_relaxed);
    }
    return c;
}

// Kernel functions whose dynamic-LDS limit has been raised: an open-addressing table of atomics, so the
// common case (already there) takes no lock; a miss takes the mutex, sets the attribute and publishes.
namespace {
constexpr int kLdsTable = 2048;
std::atomic<const void *> g_lds_done[kLdsTable];
std::mutex g_lds_mutex;
inline unsigned lds_slot(const void *fn) { return (unsigned)(((uintptr_t)fn >> 4) * 2654435761u) & (kLdsTable - 1); }
}  // namespace

bool allow_big_lds(const void *fn)
{
    if (!fn) return true;
    for (unsigned i = lds_slot(fn), n = 0; n < kLdsTable; i = (i + 1) & (kLdsTable - 1), ++n) {
        const void *e = g_lds_done[i].load(std::memory_order_acquire);
        if (e == fn) return true;
        if (!e) break;
    }
    std::lock_guard<std::mutex> lock(g_lds_mutex);
    for (unsigned i = lds_slot(fn), n = 0; n < kLdsTable; i = (i + 1) & (kLdsTable - 1), ++n) {
        const void *e = g_lds_done[i].load(std::memory_order_acquire);
        if (e == fn) return true;
        if (e) continue;
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) != hipSuccess) return false;
        g_lds_done[i].store(fn, std::memory_order_release);
        return true;
    }
    // table full (more kernels than the library has): set the attribute every time
    return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024) == hipSuccess;
}

// ---- per-launch profiler --------------------------------------------------------------
namespace {
struct ProfRecord {
    hipEvent_t start, stop;
    const char *kernel;
    const char *stage;
    double flops, bytes, mfma_flops;
};
struct ProfEntry {
    char name[96];
    long long launches;
    double ms, flops, bytes, mfma_flops;
};
thread_local ProfRecord *g_prof = nullptr;
thread_local int g_prof_cap = 0, g_prof_used = 0;
thread_local const char *g_stage = "";
thread_local ProfEntry g_entries[128];
thread_local int g_num_entries = 0;
}  // namespace

void set_stage(const char *stage) { g_stage = stage ? stage : ""; }

LaunchScope::LaunchScope(const char *kernel, double flops, double bytes, double mfma_flops) : slot(-1)
{
    if (!g_prof || g_prof_used >= g_prof_cap) return;
    slot = g_prof_used++;
    ProfRecord &r = g_prof[slot];
    r.kernel = kernel; r.stage = g_stage; r.flops = flops; r.bytes = bytes; r.mfma_flops = mfma_flops < 0 ? flops : mfma_flops;
    (void)hipEventRecord(r.start, g_stream);
}

LaunchScope::~LaunchScope()
{
    if (slot >= 0) (void)hipEventRecord(g_prof[slot].stop, g_stream);
}

int check_launch()
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        return SQ_ERR_HIP;
    }
    return SQ_OK;
}

namespace {

int out_extent(int in, int k, int s, int p) { return (in + 2 * p - k) / s + 1; }

int validate_conv(const void *in, const void *w, const float *out, int N, int Cin, int H, int W,
                  int Cout, int K, int S, int P)
{
    if (!in || !w || !out) return SQ_ERR_NULL;
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0 || K <= 0 || S < 1 || P < 0)
        return SQ_ERR_SHAPE;
    if (H + 2 * P < K || W + 2 * P < K) return SQ_ERR_SHAPE;
    return SQ_OK;
}

int run_conv(const ConvArgs &a, int algo)
{
    if (a.pool_H && (algo == SQ_ALGO_DIRECT || a.K != 1 || a.S != 1 || a.P != 0)) return SQ_ERR_UNSUPPORTED;
    if (algo == SQ_ALGO_DIRECT) return conv_direct(a);
    if (algo == SQ_ALGO_AUTO) {
        if (a.dtype == SQ_BF16 && a.ws) {   // bfloat16 operands and scratch: the bf16 matrix instructions where they pay
            const int rb = conv_bf16_mfma(a);
            if (rb != SQ_ERR_UNSUPPORTED && rb != SQ_ERR_WORKSPACE) return rb;
        }
        if (a.S >= 2 && a.ws) {   // given the scratch for it, a strided layer runs as a stride-1 one where that has a tiling
            const int rs = conv_s2d(a);
            if (rs != SQ_ERR_UNSUPPORTED) return rs;
        }
        const int rc = conv_mfma(a, -1);
        if (rc != SQ_ERR_UNSUPPORTED || a.pool_H) return rc;   // only the tiled kernels pool on the way in
        return conv_direct(a);
    }
    const int v = algo - SQ_ALGO_VARIANT0;
    if (v < 0 || v >= conv_mfma_variant_count()) return SQ_ERR_UNSUPPORTED;
    return conv_mfma(a, v);
}

ConvArgs make_args(const void *in, const void *w, const float *b, float *out, int N, int Cin, int H,
                   int W, int Cout, int K, int S, int P, int relu, int out_channels, int c_offset,
                   int dtype)
{
    ConvArgs a;
    a.in = in; a.w = w; a.b = b; a.out = out;
    a.N = N; a.Cin = Cin; a.H = H; a.W = W; a.Cout = Cout; a.K = K; a.S = S; a.P = P;
    a.relu = relu ? 1 : 0;
    a.Ho = out_extent(H, K, S, P);
    a.Wo = out_extent(W, K, S, P);
    a.out_channels = out_channels;
    a.c_offset = c_offset;
    a.dtype = dtype;
    a.ws = nullptr; a.ws_bytes = 0; a.ws_ready = false;
    a.pool_H = a.pool_W = 0;
    return a;
}

// Unchecked fire layer: squeeze into `sq_map`, then both expands into `out`.  With pool_H != 0 `in` is a
// map of pool_H x pool_W pixels that the squeeze max-pools (3x3, stride 2) down to H x W while it reads it; with
// cp_in as well, a column-pooled map of which the squeeze pools the rows.  cp_out: the expands write a column-pooled
// map for the layer behind a pooling layer; SQ_ERR_UNSUPPORTED before anything is launched where
// no kernel does that for this shape.
int fire_impl(const void *in, const void *w_sq, const float *b_sq, const void *w_e1,
              const float *b_e1, const void *w_e3, const float *b_e3, float *out, int N, int Cin,
              int H, int W, int Csq, int Ce1, int Ce3, float *sq_map, void *conv_ws, size_t conv_ws_bytes,
              bool conv_ws_ready, const char *const *stages, int pool_H = 0, int pool_W = 0, int sq_algo = SQ_ALGO_AUTO,
              const ColPool *cp_in = nullptr, const ColPool *cp_out = nullptr)
{
    ConvArgs a1 = make_args(sq_map, w_e1, b_e1, out, N, Csq, H, W, Ce1, 1, 1, 0, 1, Ce1 + Ce3, 0, SQ_F32);
    ConvArgs a3 = make_args(sq_map, w_e3, b_e3, out, N, Csq, H, W, Ce3, 3, 1, 1, 1, Ce1 + Ce3, Ce1, SQ_F32);
    a3.ws = conv_ws; a3.ws_bytes = conv_ws_bytes; a3.ws_ready = conv_ws_ready;
    if (cp_out) {
        a1.cp_out = a3.cp_out = true;
        a1.cp = a3.cp = *cp_out;
        if (!conv_expand_pair_supported(a3, a1)) return SQ_ERR_UNSUPPORTED;
    }
    set_stage(stages[0]);
    ConvArgs asq = make_args(in, w_sq, b_sq, sq_map, N, Cin, H, W, Csq, 1, 1, 0, 1, Csq, 0, SQ_F32);
    asq.pool_H = pool_H; asq.pool_W = pool_W;
    if (cp_in) {
        asq.cp_in = true;
        asq.cp = *cp_in;
    }
    int rc = run_conv(asq, sq_algo);
    if (rc) return rc;
    // Both expands in one launch: the expand1x1 tiles behind the persistent workgroups of a minimal-filtering
    // expand3x3 (batches of three images and more), else both in the tiles of one direct 3x3 kernel (small
    // batches, where a fused tiling exists for the shape), else two launches.
    set_stage(stages[3]);
    rc = conv_expand_pair(a3, a1);
    if (rc == SQ_ERR_UNSUPPORTED) rc = conv_expand_fused(a3, w_e1, b_e1, Ce1, 0);
    if (rc != SQ_ERR_UNSUPPORTED) {
        set_stage("");
        return rc;
    }
    set_stage(stages[1]);
    if ((rc = run_conv(a1, SQ_ALGO_AUTO))) return rc;
    set_stage(stages[2]);
    rc = run_conv(a3, SQ_ALGO_AUTO);
    set_stage("");
    return rc;
}

struct FireCfg { int cin, sq, e; };
const char *const kFireStages[8][4] = {
    {"fire2/sq", "fire2/e1", "fire2/e3", "fire2/e1+e3"}, {"fire3/sq", "fire3/e1", "fire3/e3", "fire3/e1+e3"},
    {"fire4/sq", "fire4/e1", "fire4/e3", "fire4/e1+e3"}, {"fire5/sq", "fire5/e1", "fire5/e3", "fire5/e1+e3"},
    {"fire6/sq", "fire6/e1", "fire6/e3", "fire6/e1+e3"}, {"fire7/sq", "fire7/e1", "fire7/e3", "fire7/e1+e3"},
    {"fire8/sq", "fire8/e1", "fire8/e3", "fire8/e1+e3"}, {"fire9/sq", "fire9/e1", "fire9/e3", "fire9/e1+e3"}};
const char *const kFireAlone[4] = {"fire/sq", "fire/e1", "fire/e3", "fire/e1+e3"};
const FireCfg kFires[8] = {{96, 16, 64},   {128, 16, 64},  {128, 32, 128}, {256, 32, 128},
                           {256, 48, 192}, {384, 48, 192}, {384, 64, 256}, {512, 64, 256}};

// Workspace carve-up of the network call: two activation buffers used in turn and
// the squeeze map.  Buffer A must hold conv1's output, buffer B the largest of the
// others (fire4's output), both per image.
constexpr size_t kBufA = (size_t)96 * 111 * 111;
constexpr size_t kBufB = (size_t)256 * 55 * 55;
constexpr size_t kBufS = (size_t)32 * 55 * 55;

int copy_tap(float *const *taps, int idx, const float *src, size_t count)
{
    if (!taps || !taps[idx]) return SQ_OK;
    const hipError_t e = hipMemcpyAsync(taps[idx], src, count * sizeof(float),
                                        hipMemcpyDeviceToDevice, current_stream());
    if (e != hipSuccess) {
        g_last_hip = (int)e;
        return SQ_ERR_HIP;
    }
    return SQ_OK;
}

}  // namespace
}  // namespace sq

using namespace sq;

extern "C" {

const char *sq_strerror(int status)
{
    switch (status) {
        case SQ_OK: return "ok";
        case SQ_ERR_NULL: return "a required pointer is NULL";
        case SQ_ERR_SHAPE: return "invalid shape, stride, padding or channel range";
        case SQ_ERR_UNSUPPORTED: return "no kernel for this dtype/algorithm/shape";
        case SQ_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case SQ_ERR_HIP: return "HIP launch failed";
        default: return "unknown status";
    }
}

int sq_last_hip_error(void) { return g_last_hip; }

int sq_set_stream(void *hip_stream)
{
    g_stream = (hipStream_t)hip_stream;
    return SQ_OK;
}

int sq_set_dtype(int dtype)
{
    if (dtype != SQ_F32 && dtype != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    g_dtype = dtype;
    return SQ_OK;
}

namespace { int static_scratch(void **ptr); }

int sq_init(void)
{
    (void)num_cus();
    void *unused = nullptr;
    const int rs = static_scratch(&unused);
    if (rs) return rs;
    const bool ok = conv_mfma_register_kernels() & blocked_register_kernels() & fire_bf16_register_kernels();
    if (!ok) {
        const int rc = check_launch();
        return rc ? rc : SQ_ERR_HIP;
    }
    return SQ_OK;
}

int sq_profile_begin(int max_launches)
{
    if (max_launches <= 0) return SQ_ERR_SHAPE;
    if (g_prof) return SQ_ERR_UNSUPPORTED;  // already profiling
    ProfRecord *recs = new ProfRecord[max_launches];
    for (int i = 0; i < max_launches; ++i) {
        if (hipEventCreate(&recs[i].start) != hipSuccess || hipEventCreate(&recs[i].stop) != hipSuccess) {
            delete[] recs;  // events made so far are left to the runtime; this path means HIP is unusable
            (void)check_launch();
            return SQ_ERR_HIP;
        }
    }
    g_prof = recs; g_prof_cap = max_launches; g_prof_used = 0; g_num_entries = 0;
    return SQ_OK;
}

int sq_profile_end(void)
{
    if (!g_prof) return SQ_ERR_UNSUPPORTED;
    int rc = SQ_OK;
    g_num_entries = 0;
    for (int i = 0; i < g_prof_used; ++i) {
        ProfRecord &r = g_prof[i];
        float ms = 0.f;
        if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) {
            rc = SQ_ERR_HIP;
            continue;
        }
        char name[96];
        snprintf(name, sizeof(name), "%s|%s", r.stage, r.kernel);
        int e = 0;
        for (; e < g_num_entries; ++e)
            if (!strcmp(g_entries[e].name, name)) break;
        if (e == g_num_entries) {
            if (g_num_entries == 128) continue;
            ++g_num_entries;
            snprintf(g_entries[e].name, sizeof(g_entries[e].name), "%s", name);
            g_entries[e].launches = 0; g_entries[e].ms = g_entries[e].flops = g_entries[e].bytes = g_entries[e].mfma_flops = 0;
        }
        g_entries[e].launches += 1; g_entries[e].ms += ms; g_entries[e].flops += r.flops; g_entries[e].bytes += r.bytes;
        g_entries[e].mfma_flops += r.mfma_flops;
    }
    for (int i = 0; i < g_prof_cap; ++i) {
        (void)hipEventDestroy(g_prof[i].start);
        (void)hipEventDestroy(g_prof[i].stop);
    }
    delete[] g_prof;
    g_prof = nullptr; g_prof_cap = g_prof_used = 0;
    if (rc) (void)check_launch();
    return rc;
}

int sq_profile_count(void) { return g_num_entries; }

int sq_profile_get(int index, char *name, int name_cap, long long *launches, double *total_ms,
                   double *flops, double *bytes)
{
    if (index < 0 || index >= g_num_entries) return SQ_ERR_SHAPE;
    if (!name || name_cap <= 0 || !launches || !total_ms || !flops || !bytes) return SQ_ERR_NULL;
    snprintf(name, (size_t)name_cap, "%s", g_entries[index].name);
    *launches = g_entries[index].launches;
    *total_ms = g_entries[index].ms;
    *flops = g_entries[index].flops;
    *bytes = g_entries[index].bytes;
    return SQ_OK;
}

int sq_profile_get_mfma_flops(int index, double *mfma_flops)
{
    if (index < 0 || index >= g_num_entries) return SQ_ERR_SHAPE;
    if (!mfma_flops) return SQ_ERR_NULL;
    *mfma_flops = g_entries[index].mfma_flops;
    return SQ_OK;
}

int sq_conv_variant_count(void) { return conv_mfma_variant_count(); }

const char *sq_conv_variant_name(int index)
{
    if (index < 0 || index >= conv_mfma_variant_count()) return "";
    return conv_mfma_variant_name(index);
}

size_t sq_conv2d_workspace_bytes(int Cin, int Cout, int K, int S, int P)
{
    if (Cin <= 0 || Cout <= 0 || K <= 0 || S < 1 || P < 0) return 0;
    return conv_workspace_bytes(Cin, Cout, K, S, P);
}

size_t sq_conv2d_strided_workspace_bytes(int N, int Cin, int H, int W, int Cout, int K, int S, int P)
{
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0 || K <= 0 || S < 1 || P < 0 || H + 2 * P < K || W + 2 * P < K) return 0;
    return conv_s2d_workspace_bytes(N, Cin, H, W, Cout, K, S, P);
}

int sq_conv2d_forward_ws(const void *in, const void *w, const float *b, float *out, int N, int Cin,
                         int H, int W, int Cout, int K, int S, int P, int relu, int out_channels,
                         int c_offset, int in_dtype, int algo, void *workspace, size_t workspace_bytes)
{
    const int rc = validate_conv(in, w, out, N, Cin, H, W, Cout, K, S, P);
    if (rc) return rc;
    if (c_offset < 0 || out_channels <= 0 || (long long)c_offset + Cout > out_channels)
        return SQ_ERR_SHAPE;
    if (in_dtype != SQ_F32 && in_dtype != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if (algo < 0) return SQ_ERR_UNSUPPORTED;
    if (workspace && ((uintptr_t)workspace & 255)) return SQ_ERR_WORKSPACE;
    ConvArgs a = make_args(in, w, b, out, N, Cin, H, W, Cout, K, S, P, relu, out_channels, c_offset, in_dtype);
    a.ws = workspace; a.ws_bytes = workspace ? workspace_bytes : 0;
    return run_conv(a, algo);
}

size_t sq_conv2d_bf16_workspace_bytes(int N, int Cin, int H, int W, int Cout, int K, int S, int P)
{
    if (S < 1) return 0;
    return conv_bf16_mfma_workspace_bytes(N, Cin, H, W, Cout, K, S, P, Cout);
}

int sq_conv2d_forward_ex(const void *in, const void *w, const float *b, float *out, int N, int Cin,
                         int H, int W, int Cout, int K, int S, int P, int relu, int out_channels,
                         int c_offset, int in_dtype, int algo)
{
    return sq_conv2d_forward_ws(in, w, b, out, N, Cin, H, W, Cout, K, S, P, relu, out_channels, c_offset,
                                in_dtype, algo, nullptr, 0);
}

int sq_conv2d_forward(const void *in, const void *w, const float *b, float *out, int N, int Cin,
                      int H, int W, int Cout, int K, int S, int P, int relu)
{
    return sq_conv2d_forward_ex(in, w, b, out, N, Cin, H, W, Cout, K, S, P, relu, Cout, 0, g_dtype,
                                SQ_ALGO_AUTO);
}

int sq_maxpool_conv2d_forward(const float *in, const float *w, const float *b, float *out, int N, int Cin, int H,
                              int W, int Cout, int relu, int out_channels, int c_offset, int algo)
{
    if (!in || !w || !out) return SQ_ERR_NULL;
    if (N <= 0 || Cin <= 0 || Cout <= 0 || H < 3 || W < 3) return SQ_ERR_SHAPE;
    if (c_offset < 0 || out_channels <= 0 || (long long)c_offset + Cout > out_channels) return SQ_ERR_SHAPE;
    if (algo < 0 || algo == SQ_ALGO_DIRECT) return SQ_ERR_UNSUPPORTED;
    const int Hp = (H - 3) / 2 + 1, Wp = (W - 3) / 2 + 1;
    ConvArgs a = make_args(in, w, b, out, N, Cin, Hp, Wp, Cout, 1, 1, 0, relu, out_channels, c_offset, SQ_F32);
    a.pool_H = H; a.pool_W = W;
    return run_conv(a, algo);
}

// ---- the kernels of the split pooling one at a time (tests, tuner; declared in sq_tuning.h) -----------------
int sq_tune_conv2d_forward_poolcols(const float *in, const float *w, const float *b, float *out, int N, int Cin, int H, int W,
                                    int Cout, int K, int S, int P, int *geometry)
{
    if (!in || !w || !out || !geometry) return SQ_ERR_NULL;
    if (N <= 0 || H <= 0 || W <= 0 || P < 0) return SQ_ERR_SHAPE;
    if (Cin != 3 || K != 7 || S != 2 || Cout != 96 || g_dtype != SQ_F32) return SQ_ERR_UNSUPPORTED;
    if (H + 2 * P < K || W + 2 * P < K) return SQ_ERR_SHAPE;
    ConvArgs a = make_args(in, w, b, out, N, Cin, H, W, Cout, K, S, P, 1, Cout, 0, SQ_F32);
    if (a.Wo < 3) return SQ_ERR_SHAPE;
    // tiles of 2 rows x 16 columns = 8 pooled columns
    const int CB = (a.Wo + 15) / 16, RG = (a.Ho + 1) / 2;
    a.cp_out = true;
    a.cp.shift = 3; a.cp.slots_row = 8 * CB; a.cp.slots_image = 8 * CB * RG;
    a.cp.row_stride = colpool_row_stride(a.Wo, 3);
    geometry[0] = a.cp.shift; geometry[1] = a.cp.slots_row; geometry[2] = a.cp.slots_image; geometry[3] = a.cp.row_stride;
    return conv_mfma(a, -1);
}

int sq_tune_fire_forward_poolcols(const float *in, const float *w_sq, const float *b_sq, const float *w_e1, const float *b_e1,
                                  const float *w_e3, const float *b_e3, float *out, int N, int Cin, int H, int W, int Csq,
                                  int Ce1, int Ce3, void *workspace, size_t workspace_bytes, int *geometry)
{
    if (!in || !w_sq || !w_e1 || !w_e3 || !out || !geometry) return SQ_ERR_NULL;
    if (N <= 0 || Cin <= 0 || H <= 0 || W < 3 || Csq <= 0 || Ce1 <= 0 || Ce3 <= 0) return SQ_ERR_SHAPE;
    if (g_dtype != SQ_F32) return SQ_ERR_UNSUPPORTED;
    const size_t map_bytes = align_up((size_t)N * Csq * H * W * sizeof(float), 256);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < sq_fire_workspace_bytes(N, H, W, Csq, Ce3)) return SQ_ERR_WORKSPACE;
    // tile groups of the expand pair: 16 tiles of 2 x 2 pixels, numbered through the batch
    ColPool cp;
    cp.shift = 4; cp.slots_row = (W + 1) / 2; cp.slots_image = cp.slots_row * ((H + 1) / 2);
    cp.row_stride = colpool_row_stride(W, 4);
    geometry[0] = cp.shift; geometry[1] = cp.slots_row; geometry[2] = cp.slots_image; geometry[3] = cp.row_stride;
    return fire_impl(in, w_sq, b_sq, w_e1, b_e1, w_e3, b_e3, out, N, Cin, H, W, Csq, Ce1, Ce3, (float *)workspace,
                     (char *)workspace + map_bytes, workspace_bytes - map_bytes, false, kFireAlone, 0, 0, SQ_ALGO_AUTO, nullptr, &cp);
}

int sq_tune_poolrows_conv2d_forward(const float *in, const float *w, const float *b, float *out, int N, int Cin, int H, int W,
                                    int Cout, int relu, int out_channels, int c_offset, int algo, const int *geometry)
{
    if (!in || !w || !out || !geometry) return SQ_ERR_NULL;
    if (N <= 0 || Cin <= 0 || Cout <= 0 || H < 3 || W < 3) return SQ_ERR_SHAPE;
    if (c_offset < 0 || out_channels <= 0 || (long long)c_offset + Cout > out_channels) return SQ_ERR_SHAPE;
    if (algo < 0 || algo == SQ_ALGO_DIRECT || g_dtype != SQ_F32) return SQ_ERR_UNSUPPORTED;
    const int Hp = (H - 3) / 2 + 1, Wp = (W - 3) / 2 + 1;
    // the geometry must describe rows of (W + 1) / 2 or more slots that hold every seam
    if (geometry[0] < 1 || geometry[0] > 8 || geometry[1] < Wp || geometry[2] < geometry[1] * ((H + 1) / 2) ||
        geometry[3] < colpool_row_stride(W, geometry[0]) || (long long)N * geometry[2] >= (1ll << 30))
        return SQ_ERR_SHAPE;
    ConvArgs a = make_args(in, w, b, out, N, Cin, Hp, Wp, Cout, 1, 1, 0, relu, out_channels, c_offset, SQ_F32);
    a.pool_H = H; a.pool_W = W;
    a.cp_in = true;
    a.cp.shift = geometry[0]; a.cp.slots_row = geometry[1]; a.cp.slots_image = geometry[2]; a.cp.row_stride = geometry[3];
    return run_conv(a, algo);
}

int sq_maxpool(const float *in, float *out, int N, int C, int H, int W, int K, int S)
{
    if (!in || !out) return SQ_ERR_NULL;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || S < 1 || K > H || K > W) return SQ_ERR_SHAPE;
    return maxpool(in, out, N, C, H, W, K, S);
}

int sq_avgpool_global(const float *in, float *out, int N, int C, int H, int W)
{
    if (!in || !out) return SQ_ERR_NULL;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return SQ_ERR_SHAPE;
    return avgpool_global(in, out, N, C, H, W);
}

int sq_softmax(const float *in, float *out, int N, int C)
{
    if (!in || !out) return SQ_ERR_NULL;
    if (N <= 0 || C <= 0) return SQ_ERR_SHAPE;
    return softmax(in, out, N, C);
}

size_t sq_classifier_workspace_bytes(int N, int Cin, int H, int W, int Cout)
{
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0) return 0;
    // room for either form: the plane sums of the fused form, or the map and the means of the three separate layers
    const ConvArgs a = make_args((const void *)256, (const void *)256, nullptr, (float *)256, N, Cin, H, W, Cout, 1, 1, 0, 1, Cout, 0, SQ_F32);
    const size_t fused = conv_mfma_avg_bytes(a, -1);
    const size_t plain = align_up((size_t)N * Cout * H * W * sizeof(float), 256) + align_up((size_t)N * Cout * sizeof(float), 256);
    return align_up(fused > plain ? fused : plain, 256);
}

int sq_classifier_forward(const float *in, const float *w, const float *b, float *means, float *probs, int N, int Cin, int H,
                          int W, int Cout, void *workspace, size_t workspace_bytes)
{
    if (!in || !w || !probs) return SQ_ERR_NULL;
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0) return SQ_ERR_SHAPE;
    if (g_dtype != SQ_F32) return SQ_ERR_UNSUPPORTED;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < sq_classifier_workspace_bytes(N, Cin, H, W, Cout))
        return SQ_ERR_WORKSPACE;
    ConvArgs a = make_args(in, w, b, (float *)workspace, N, Cin, H, W, Cout, 1, 1, 0, 1, Cout, 0, SQ_F32);
    AvgLayout lay;
    set_stage("classifier/conv");
    int rc = (g_fuse_classifier < 0 ? N >= 8 : g_fuse_classifier) ? conv_mfma_avg(a, -1, (float *)workspace, workspace_bytes, &lay)
                                                                   : (int)SQ_ERR_UNSUPPORTED;
    if (rc == SQ_OK) {
        set_stage("classifier/avgpool+softmax");
        rc = avg_softmax((const float *)workspace, lay, means, probs, N, Cout, H * W);
        if (rc != SQ_ERR_UNSUPPORTED) {
            set_stage("");
            return rc;
        }
    }
    if (rc != SQ_ERR_UNSUPPORTED) {
        set_stage("");
        return rc;
    }
    // the three layers one after the other
    float *map = (float *)workspace;
    float *mean_buf = means ? means : (float *)((char *)workspace + align_up((size_t)N * Cout * H * W * sizeof(float), 256));
    if (!(rc = run_conv(a, SQ_ALGO_AUTO))) {
        set_stage("classifier/avgpool");
        if (!(rc = avgpool_global(map, mean_buf, N, Cout, H, W))) {
            set_stage("classifier/softmax");
            rc = softmax(mean_buf, probs, N, Cout);
        }
    }
    set_stage("");
    return rc;
}

size_t sq_fire_workspace_bytes(int N, int H, int W, int Csq, int Ce3)
{
    if (N <= 0 || H <= 0 || W <= 0 || Csq <= 0 || Ce3 <= 0) return 0;
    return align_up((size_t)N * Csq * H * W * sizeof(float), 256) + conv_workspace_bytes(Csq, Ce3, 3, 1, 1);
}

namespace {
// packed_e3: the expand3x3 kernels as sq_fire_pack_weights wrote them, or nullptr = transform them into the workspace
int fire_checked(const void *in, const void *w_sq, const float *b_sq, const void *w_e1, const float *b_e1, const void *w_e3,
                 const float *b_e3, const void *packed_e3, float *out, int N, int Cin, int H, int W, int Csq, int Ce1, int Ce3,
                 void *workspace, size_t workspace_bytes)
{
    if (!in || !w_sq || !w_e1 || !w_e3 || !out) return SQ_ERR_NULL;
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Csq <= 0 || Ce1 <= 0 || Ce3 <= 0) return SQ_ERR_SHAPE;
    if (g_dtype != SQ_F32) return SQ_ERR_UNSUPPORTED;   // the reduced-precision fire layer is sq_blocked_fire_forward
    const size_t map_bytes = align_up((size_t)N * Csq * H * W * sizeof(float), 256);
    const size_t need = packed_e3 ? map_bytes : sq_fire_workspace_bytes(N, H, W, Csq, Ce3);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < need) return SQ_ERR_WORKSPACE;
    if (packed_e3 && ((uintptr_t)packed_e3 & 255)) return SQ_ERR_WORKSPACE;
    if (packed_e3)
        return fire_impl(in, w_sq, b_sq, w_e1, b_e1, w_e3, b_e3, out, N, Cin, H, W, Csq, Ce1, Ce3, (float *)workspace,
                         const_cast<void *>(packed_e3), conv_workspace_bytes(Csq, Ce3, 3, 1, 1), true, kFireAlone);
    return fire_impl(in, w_sq, b_sq, w_e1, b_e1, w_e3, b_e3, out, N, Cin, H, W, Csq, Ce1, Ce3, (float *)workspace,
                     (char *)workspace + map_bytes, workspace_bytes - map_bytes, false, kFireAlone);
}
}  // namespace

int sq_fire_forward(const void *in, const void *w_sq, const float *b_sq, const void *w_e1,
                    const float *b_e1, const void *w_e3, const float *b_e3, float *out, int N,
                    int Cin, int H, int W, int Csq, int Ce1, int Ce3, void *workspace,
                    size_t workspace_bytes)
{
    return fire_checked(in, w_sq, b_sq, w_e1, b_e1, w_e3, b_e3, nullptr, out, N, Cin, H, W, Csq, Ce1, Ce3, workspace,
                        workspace_bytes);
}

// ---- the fire layer for callers that cannot allocate: scratch in a static device array ---------------------
// Every GPU the library runs on holds its own copy of the array, at its own address, until the process ends.
// In host code the array's name is only a handle: its device address is asked for once per device (with that
// device current) and kept; the kernels get that address as an argument, as they get a caller's workspace.
namespace {
__device__ __align__(256) unsigned char scratch[SQ_FIRE_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

int static_scratch(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        const int rc = check_launch();
        return rc ? rc : SQ_ERR_HIP;
    }
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        p = g_scratch_ptr[dev].load(std::memory_order_acquire);
        if (!p) {
            if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
                const int rc = check_launch();
                return rc ? rc : SQ_ERR_HIP;
            }
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *ptr = p;
    return SQ_OK;
}
}  // namespace

int sq_fire_forward_static(const void *in, const void *w_sq, const float *b_sq, const void *w_e1, const float *b_e1,
                           const void *w_e3, const float *b_e3, float *out, int N, int Cin, int H, int W, int Csq, int Ce1,
                           int Ce3)
{
    if (!in || !w_sq || !w_e1 || !w_e3 || !out) return SQ_ERR_NULL;
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Csq <= 0 || Ce1 <= 0 || Ce3 <= 0) return SQ_ERR_SHAPE;
    // the sizes are checked in 64 bits before anything else: a layer beyond the array is refused, never truncated
    const unsigned long long map = ((unsigned long long)N * Csq * H * W * sizeof(float) + 255) / 256 * 256;
    if (map > SQ_FIRE_STATIC_SCRATCH_BYTES || map + conv_workspace_bytes(Csq, Ce3, 3, 1, 1) > SQ_FIRE_STATIC_SCRATCH_BYTES)
        return SQ_ERR_WORKSPACE;
    void *ptr = nullptr;
    const int rc = static_scratch(&ptr);
    if (rc) return rc;
    return fire_checked(in, w_sq, b_sq, w_e1, b_e1, w_e3, b_e3, nullptr, out, N, Cin, H, W, Csq, Ce1, Ce3, ptr,
                        SQ_FIRE_STATIC_SCRATCH_BYTES);
}

size_t sq_fire_packed_bytes(int Csq, int Ce3)
{
    if (Csq <= 0 || Ce3 <= 0) return 0;
    return conv_workspace_bytes(Csq, Ce3, 3, 1, 1);
}

int sq_fire_pack_weights(const void *w_e3, void *packed, size_t packed_bytes, int Csq, int Ce3)
{
    if (!w_e3 || !packed) return SQ_ERR_NULL;
    if (Csq <= 0 || Ce3 <= 0) return SQ_ERR_SHAPE;
    const size_t need = conv_workspace_bytes(Csq, Ce3, 3, 1, 1);
    if (!need) return SQ_ERR_UNSUPPORTED;   // this shape has no packed form: call sq_fire_forward
    if (((uintptr_t)packed & 255) || packed_bytes < need) return SQ_ERR_WORKSPACE;
    const KernelPrepJob job{w_e3, packed, Csq, Ce3};
    set_stage("kernel transform");
    const int rc = conv_prepare_kernels(&job, 1, SQ_F32);
    set_stage("");
    return rc;
}

int sq_fire_forward_packed(const void *in, const void *w_sq, const float *b_sq, const void *w_e1, const float *b_e1,
                           const void *w_e3, const float *b_e3, const void *packed_e3, float *out, int N, int Cin, int H, int W,
                           int Csq, int Ce1, int Ce3, void *workspace, size_t workspace_bytes)
{
    if (!packed_e3) return SQ_ERR_NULL;
    if (Csq > 0 && Ce3 > 0 && !conv_workspace_bytes(Csq, Ce3, 3, 1, 1)) return SQ_ERR_UNSUPPORTED;
    return fire_checked(in, w_sq, b_sq, w_e1, b_e1, w_e3, b_e3, packed_e3, out, N, Cin, H, W, Csq, Ce1, Ce3, workspace,
                        workspace_bytes);
}

size_t sq_squeezenet_workspace_bytes(int N)
{
    if (N <= 0) return 0;
    const size_t n = (size_t)N;
    size_t conv_ws = 0;   // every expand3x3 layer has its own area: all are filled by one launch
    for (const FireCfg &fc : kFires) conv_ws += conv_workspace_bytes(fc.sq, fc.e, 3, 1, 1);
    return align_up(n * kBufA * 4, 256) + align_up(n * kBufB * 4, 256) + align_up(n * kBufS * 4, 256) +
           align_up(n * 1000 * 4, 256) + conv_ws;
}

// Which max-pooling layers of the fp32 network run inside the squeeze layer that reads them: bit 0 = pool1,
// bit 1 = pool4, bit 2 = pool8; bits 3..5 = the same three, split between the layer before (columns) and the
// squeeze (rows); -1 = the default policy: what made the whole pass faster when measured at batches 1 to 256.
// Inside the squeeze: pool1 everywhere; pool4 from batch 4 on (below that the squeeze of fire5 has too few
// workgroups to hide nine loads per element); pool8 from batch 64 on.  Split: all three from batch 64 on, where the
// maps no longer stay in the memory-side cache between two layers and bytes count (whole pass 1010 -> 970 us at
// batch 64, 1964 -> 1823 at 128, 3853 -> 3675 at 256; at batch 32 and below the split changes nothing or costs
// 1-2 %: conv1 pays 8 % for the column maxima).  A call with taps keeps every pooled map, but runs the squeeze with
// the tiling the fused forms would use, so the results are the same bit for bit.
// The setter is a tuning hook, not part of the public interface.
extern "C" void sq_tune_fuse_classifier(int on) { g_fuse_classifier = on < 0 ? -1 : on ? 1 : 0; }
thread_local int g_fuse_pools_f32 = -1;
extern "C" void sq_tune_fuse_pools_f32(int mask) { g_fuse_pools_f32 = mask; }
int fuse_pools_f32_policy(int N) { return 1 | (N >= 4 ? 2 : 0) | (N >= 64 ? 4 : 0) | (N >= 64 ? 56 : 0); }

namespace {
size_t packed_f32_bytes()
{
    size_t b = 0;
    for (const FireCfg &fc : kFires) b += conv_workspace_bytes(fc.sq, fc.e, 3, 1, 1);
    return b;
}
}  // namespace

// packed: the expand3x3 kernels of the eight fire layers as sq_pack_weights(SQ_F32) wrote them, or nullptr = they
// are transformed into the workspace by one launch at the start of the call.
static int squeezenet_f32(const void *in, const void *const *params, const void *packed, float *probs, int N,
                          void *workspace, size_t workspace_bytes, float *const *taps)
{
    if (!in || !params || !probs) return SQ_ERR_NULL;
    if (N <= 0) return SQ_ERR_SHAPE;
    if (N > SQ_SQUEEZENET_MAX_BATCH) return SQ_ERR_UNSUPPORTED;   // conv1's output would pass 2^29 elements
    for (int i = 0; i < 52; ++i)
        if (!params[i]) return SQ_ERR_NULL;
    if (taps && taps[15]) return SQ_ERR_UNSUPPORTED;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < sq_squeezenet_workspace_bytes(N))
        return SQ_ERR_WORKSPACE;

    const size_t n = (size_t)N;
    char *base = (char *)workspace;
    float *bufA = (float *)base;
    float *bufB = (float *)(base + align_up(n * kBufA * 4, 256));
    float *bufS = (float *)((char *)bufB + align_up(n * kBufB * 4, 256));
    float *means = (float *)((char *)bufS + align_up(n * kBufS * 4, 256));
    auto P = [&](int i) { return (const float *)params[i]; };
    // transformed kernels of those expand3x3 layers whose algorithm wants them, written by
    // one launch up front
    char *conv_ws[8];
    size_t conv_ws_bytes[8];
    bool conv_ws_ready[8];
    KernelPrepJob prep[8];
    int nprep = 0;
    {
        char *next = packed ? (char *)const_cast<void *>(packed) : (char *)means + align_up(n * 1000 * 4, 256);
        int h = 55;
        for (int f = 0; f < 8; ++f) {
            const FireCfg &fc = kFires[f];
            conv_ws[f] = next;
            conv_ws_bytes[f] = conv_workspace_bytes(fc.sq, fc.e, 3, 1, 1);
            next += conv_ws_bytes[f];
            ConvArgs a3 = make_args(bufS, params[2 + 6 * f + 4], nullptr, bufA, N, fc.sq, h, h, fc.e, 3, 1, 1, 1,
                                    2 * fc.e, fc.e, SQ_F32);
            a3.ws = conv_ws[f]; a3.ws_bytes = conv_ws_bytes[f];
            conv_ws_ready[f] = packed != nullptr || conv_wants_prepared_kernels(a3, true);
            if (conv_ws_ready[f] && !packed) prep[nprep++] = KernelPrepJob{params[2 + 6 * f + 4], conv_ws[f], fc.sq, fc.e};
            if (f == 2) h = 27;
            if (f == 6) h = 13;
        }
    }
    int rc = SQ_OK;
    if (nprep && !packed) {
        set_stage("kernel transform");
        if ((rc = conv_prepare_kernels(prep, nprep, SQ_F32))) return rc;
    }
    // Pooling layers (bits 0..2 = pool1, pool4, pool8): `inside` = pooled by the squeeze that reads the map (nine loads
    // per element of the full map), `split` = columns pooled by the layer before, rows by that squeeze (ColPool: half
    // the bytes written and read); a split that has no kernel for its shape falls back to `inside`.  A call with
    // taps keeps every map, but runs the squeezes with the tiling the fused forms would use: same bits either way.
    const int mask = g_fuse_pools_f32 >= 0 ? g_fuse_pools_f32 : fuse_pools_f32_policy(N);
    const int pools_in_squeeze = (mask | (mask >> 3)) & 7;
    const int fuse_pools = taps ? 0 : pools_in_squeeze;
    const int split_pools = taps ? 0 : (mask >> 3) & 7;
    ColPool cp_pending;          // geometry of the column-pooled map `cur`, if it is one
    bool cp_is_pending = false;
    auto colpool_of = [&](int shift, int slots_row, int rows, int Wo) {
        ColPool cp;
        cp.shift = shift; cp.slots_row = slots_row; cp.slots_image = slots_row * rows;
        cp.row_stride = colpool_row_stride(Wo, shift);
        return cp;
    };
    set_stage("conv1");
    ConvArgs a_conv1 = make_args(in, params[0], P(1), bufA, N, 3, 224, 224, 96, 7, 2, 2, 1, 96, 0, SQ_F32);
    if (split_pools & 1) {
        // conv1 tiles: 2 rows x 16 columns = 8 pooled columns, 56 x 7 per image
        ConvArgs c = a_conv1;
        c.cp_out = true;
        c.cp = colpool_of(3, 56, 56, 111);
        if (conv_mfma_choice(c) >= 0) {
            a_conv1 = c;
            cp_pending = c.cp;
            cp_is_pending = true;
        }
    }
    rc = run_conv(a_conv1, SQ_ALGO_AUTO);
    if (rc) return rc;
    if ((rc = copy_tap(taps, 0, bufA, n * 96 * 111 * 111))) return rc;
    // tiling of the squeeze behind pool `bit` when the pooled map is kept although the policy would not keep it
    auto squeeze_algo = [&](int bit, int f, int C, int H_in) {
        if (!(pools_in_squeeze & bit) || (fuse_pools & bit)) return (int)SQ_ALGO_AUTO;
        const int Hp = (H_in - 3) / 2 + 1;
        ConvArgs a = make_args(bufA, params[2 + 6 * f], nullptr, bufS, N, C, Hp, Hp, kFires[f].sq, 1, 1, 0, 1, kFires[f].sq, 0, SQ_F32);
        a.pool_H = a.pool_W = H_in;
        const int v = conv_mfma_choice(a);
        return v >= 0 ? SQ_ALGO_VARIANT0 + v : (int)SQ_ALGO_AUTO;
    };
    float *cur = bufA, *nxt = bufB;
    int pooled_from = 0;   // extent of the map `cur` before the pooling that the next squeeze is to do, or 0
    int sq_algo = squeeze_algo(1, 0, 96, 111);
    if (fuse_pools & 1) {
        pooled_from = 111;
    } else {
        set_stage("pool1");
        if ((rc = maxpool(bufA, bufB, N, 96, 111, 111, 3, 2))) return rc;
        if ((rc = copy_tap(taps, 1, bufB, n * 96 * 55 * 55))) return rc;
        cur = bufB; nxt = bufA;
    }

    int C = 96, H = 55, tap = 2, p = 2;
    for (int f = 0; f < 8; ++f) {
        const FireCfg &fc = kFires[f];
        // Only the squeeze reads a fire layer's input, and it has finished before the expands start.  A layer
        // that pools on the way in therefore writes over its own input: every later layer then finds its
        // input and output in the same buffer as without the fusion (with the roles exchanged instead, conv1
        // and several later layers ran measurably slower at batch 32).
        float *dst = pooled_from ? cur : nxt;
        const bool pool_behind = f == 2 || f == 6;    // pooling follows fire4 and fire8
        const int pool_bit = f == 2 ? 2 : 4;
        const ColPool cp_in = cp_pending;
        const bool has_cp_in = cp_is_pending;
        cp_is_pending = false;
        rc = SQ_ERR_UNSUPPORTED;
        if (pool_behind && (split_pools & pool_bit)) {
            // tile groups of the expand pair: 16 tiles of 2 x 2 pixels in a row of (H + 1) / 2, numbered through the batch
            const int TX = (H + 1) / 2;
            const ColPool cp_out = colpool_of(4, TX, TX, H);
            rc = fire_impl(cur, params[p], P(p + 1), params[p + 2], P(p + 3), params[p + 4], P(p + 5), dst,
                           N, C, H, H, fc.sq, fc.e, fc.e, bufS, conv_ws[f], conv_ws_bytes[f], conv_ws_ready[f], kFireStages[f],
                           pooled_from, pooled_from, sq_algo, has_cp_in ? &cp_in : nullptr, &cp_out);
            if (rc == SQ_OK) {
                cp_pending = cp_out;
                cp_is_pending = true;
            }
        }
        if (rc == SQ_ERR_UNSUPPORTED)
            rc = fire_impl(cur, params[p], P(p + 1), params[p + 2], P(p + 3), params[p + 4], P(p + 5), dst,
                           N, C, H, H, fc.sq, fc.e, fc.e, bufS, conv_ws[f], conv_ws_bytes[f], conv_ws_ready[f], kFireStages[f],
                           pooled_from, pooled_from, sq_algo, has_cp_in ? &cp_in : nullptr, nullptr);
        sq_algo = SQ_ALGO_AUTO;
        if (rc) return rc;
        p += 6;
        C = 2 * fc.e;
        if ((rc = copy_tap(taps, tap++, dst, n * C * H * H))) return rc;
        if (!pooled_from) { float *t = cur; cur = nxt; nxt = t; }
        pooled_from = 0;
        if (pool_behind) {
            sq_algo = squeeze_algo(pool_bit, f + 1, C, H);
            if (fuse_pools & pool_bit) {
                pooled_from = H;
                H = (H - 3) / 2 + 1;
                ++tap;
                continue;
            }
            set_stage(f == 2 ? "pool4" : "pool8");
            if ((rc = maxpool(cur, nxt, N, C, H, H, 3, 2))) return rc;
            H = (H - 3) / 2 + 1;
            if ((rc = copy_tap(taps, tap++, nxt, n * C * H * H))) return rc;
            { float *t = cur; cur = nxt; nxt = t; }
        }
    }
    // conv10 -> global average pooling -> softmax.  The convolution writes per-image plane sums of its results instead
    // of the 1000 x 13 x 13 map (which is then never written or read), and one more launch turns them into class means
    // and probabilities.  A caller who wants to see the map gets it from an extra, plain run of the convolution; means
    // and probabilities come from the same two launches either way, so taps do not change them.
    const ConvArgs a10 = make_args(cur, params[50], P(51), nxt, N, 512, H, H, 1000, 1, 1, 0, 1, 1000, 0, SQ_F32);
    set_stage("conv10");
    bool have_map = false;
    if (taps && taps[12]) {
        if ((rc = run_conv(a10, SQ_ALGO_AUTO))) return rc;
        if ((rc = copy_tap(taps, 12, nxt, n * 1000 * H * H))) return rc;
        have_map = true;
    }
    AvgLayout lay;
    rc = (g_fuse_classifier < 0 ? N >= 8 : g_fuse_classifier) ? conv_mfma_avg(a10, -1, bufS, n * kBufS * 4, &lay) : (int)SQ_ERR_UNSUPPORTED;
    if (rc == SQ_OK) {
        set_stage("avgpool+softmax");
        if ((rc = avg_softmax(bufS, lay, means, probs, N, 1000, H * H))) return rc;
    } else if (rc == SQ_ERR_UNSUPPORTED || rc == SQ_ERR_WORKSPACE) {
        if (!have_map && (rc = run_conv(a10, SQ_ALGO_AUTO))) return rc;
        set_stage("avgpool");
        if ((rc = avgpool_global(nxt, means, N, 1000, H, H))) return rc;
        set_stage("softmax");
        if ((rc = softmax(means, probs, N, 1000))) return rc;
    } else {
        return rc;
    }
    set_stage("");
    if ((rc = copy_tap(taps, 13, means, n * 1000))) return rc;
    return copy_tap(taps, 14, probs, n * 1000);
}

int sq_squeezenet_forward(const void *in, const void *const *params, float *probs, int N,
                          void *workspace, size_t workspace_bytes, float *const *taps)
{
    if (g_dtype != SQ_F32) return SQ_ERR_UNSUPPORTED;   // reduced precision needs packed kernels: sq_squeezenet_forward_packed
    return squeezenet_f32(in, params, nullptr, probs, N, workspace, workspace_bytes, taps);
}

size_t sq_packed_weights_bytes(int dtype)
{
    if (dtype == SQ_F32) return packed_f32_bytes();
    if (dtype == SQ_BF16) return sq_squeezenet_bf16_packed_bytes();
    return 0;
}

int sq_pack_weights(const void *const *params, int dtype, void *packed, size_t packed_bytes)
{
    if (dtype == SQ_BF16) return sq_squeezenet_bf16_pack_params(params, packed, packed_bytes);
    if (dtype != SQ_F32) return SQ_ERR_UNSUPPORTED;
    if (!params || !packed) return SQ_ERR_NULL;
    for (int i = 0; i < 52; ++i)
        if (!params[i]) return SQ_ERR_NULL;
    if (((uintptr_t)packed & 255) || packed_bytes < packed_f32_bytes()) return SQ_ERR_WORKSPACE;
    KernelPrepJob prep[8];
    char *next = (char *)packed;
    for (int f = 0; f < 8; ++f) {
        prep[f] = KernelPrepJob{params[2 + 6 * f + 4], next, kFires[f].sq, kFires[f].e};
        next += conv_workspace_bytes(kFires[f].sq, kFires[f].e, 3, 1, 1);
    }
    set_stage("kernel transform");
    const int rc = conv_prepare_kernels(prep, 8, SQ_F32);
    set_stage("");
    return rc;
}

int sq_squeezenet_forward_packed(const void *in, const void *const *params, const void *packed, float *probs, int N,
                                 void *workspace, size_t workspace_bytes, float *const *taps)
{
    if (!packed) return SQ_ERR_NULL;
    if ((uintptr_t)packed & 255) return SQ_ERR_WORKSPACE;
    if (g_dtype == SQ_BF16)
        return sq_squeezenet_forward_bf16(in, SQ_F32, params, packed, probs, N, workspace, workspace_bytes, taps);
    return squeezenet_f32(in, params, packed, probs, N, workspace, workspace_bytes, taps);
}

// ---- reduced-precision path on blocked bfloat16 maps -------------------------------------
size_t sq_blocked_map_bytes(int N, int C, int H, int W)
{
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return 0;
    return blocked_map_bytes(N, C, H, W);
}

int sq_blocked_pack(const void *in, sq_dtype in_dtype, void *out, int N, int C, int H, int W)
{
    if (!in || !out) return SQ_ERR_NULL;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return SQ_ERR_SHAPE;
    if (in_dtype != SQ_F32 && in_dtype != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    return blocked_pack_map(in, in_dtype, out, N, C, H, W);
}

int sq_blocked_unpack(const void *in, float *out, int N, int C, int H, int W)
{
    if (!in || !out) return SQ_ERR_NULL;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return SQ_ERR_SHAPE;
    return blocked_unpack_map(in, out, N, C, H, W);
}

size_t sq_blocked_kernel_bytes(int Cout, int Cin, int K)
{
    if (Cout <= 0 || Cin <= 0 || K <= 0) return 0;
    return blocked_packed_kernel_bytes(Cout, Cin, K);
}

int sq_blocked_pack_kernels(const void *w, sq_dtype w_dtype, void *packed, int Cout, int Cin, int K)
{
    if (!w || !packed) return SQ_ERR_NULL;
    if (Cout <= 0 || Cin <= 0 || K <= 0) return SQ_ERR_SHAPE;
    if (w_dtype != SQ_F32 && w_dtype != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if ((uintptr_t)packed & 15) return SQ_ERR_UNSUPPORTED;
    return blocked_pack_kernels(w, w_dtype, packed, Cout, Cin, K);
}

int sq_blocked_conv2d_forward(const void *in, const void *packed_w, const float *b, void *out, int N, int Cin, int H,
                              int W, int Cout, int K, int P, int relu, int ldc_channels, int c_offset)
{
    if (!in || !packed_w || !out) return SQ_ERR_NULL;
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Cout <= 0 || K <= 0 || P < 0) return SQ_ERR_SHAPE;
    if (c_offset < 0 || ldc_channels < c_offset + Cout) return SQ_ERR_SHAPE;
    if (((uintptr_t)in & 15) || ((uintptr_t)out & 15) || ((uintptr_t)packed_w & 15)) return SQ_ERR_UNSUPPORTED;
    return blocked_conv(in, packed_w, b, out, N, Cin, H, W, Cout, K, P, relu ? 1 : 0, ldc_channels, c_offset);
}

size_t sq_blocked_kernel7_bytes(void) { return blocked_packed_kernel7_bytes(); }

int sq_blocked_pack_kernels7(const void *w, sq_dtype w_dtype, void *packed, int Cout)
{
    if (!w || !packed) return SQ_ERR_NULL;
    if (Cout <= 0) return SQ_ERR_SHAPE;
    if (w_dtype != SQ_F32 && w_dtype != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if ((uintptr_t)packed & 15) return SQ_ERR_UNSUPPORTED;
    return blocked_pack_kernels7(w, w_dtype, packed, Cout);
}

int sq_blocked_conv7s2_forward(const void *in, sq_dtype in_dtype, const void *packed_w, const float *b, void *out, int N,
                               int H, int W, int Cout, int P, int relu, int ldc_channels, int c_offset)
{
    if (!in || !packed_w || !out) return SQ_ERR_NULL;
    if (N <= 0 || H <= 0 || W <= 0 || Cout <= 0 || P < 0 || H + 2 * P < 7 || W + 2 * P < 7) return SQ_ERR_SHAPE;
    if (c_offset < 0 || ldc_channels < c_offset + Cout) return SQ_ERR_SHAPE;
    if (in_dtype != SQ_F32 && in_dtype != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if (((uintptr_t)out & 15) || ((uintptr_t)packed_w & 15)) return SQ_ERR_UNSUPPORTED;
    return blocked_conv7s2(in, in_dtype, packed_w, b, out, N, H, W, Cout, P, relu ? 1 : 0, ldc_channels, c_offset);
}

int sq_blocked_pool_conv2d_forward(const void *in, const void *packed_w, const float *b, void *out, int N, int Cin, int Hin,
                                   int Win, int Cout, int relu, int ldc_channels, int c_offset)
{
    if (!in || !packed_w || !out) return SQ_ERR_NULL;
    if (N <= 0 || Cin <= 0 || Hin < 3 || Win < 3 || Cout <= 0) return SQ_ERR_SHAPE;
    if (c_offset < 0 || ldc_channels < c_offset + Cout) return SQ_ERR_SHAPE;
    if (((uintptr_t)in & 15) || ((uintptr_t)out & 15) || ((uintptr_t)packed_w & 15)) return SQ_ERR_UNSUPPORTED;
    return blocked_pool_conv(in, packed_w, b, out, N, Cin, Hin, Win, Cout, relu ? 1 : 0, ldc_channels, c_offset);
}

// Whether a reduced-precision fire layer runs as one launch (squeeze map kept in LDS): 1 = always where the
// shape is covered, 0 = never, -1 = the default policy by batch size.  Tuning hook, not part of the interface.
// Measured on MI355X the one launch is slower than squeeze + paired expands at every batch (network pass at
// batch 1 / 2 / 4 / 8 / 16: 0.133 / 0.143 / 0.154 / 0.185 / 0.261 ms against 0.124 / 0.129 / 0.140 / 0.156 /
// 0.179 ms): with a band of a few rows per workgroup only two or three of its eight wavefronts have a pixel
// block in each phase, and each walks its 6 to 36 dependent steps alone.  So the policy never picks it; it
// stays selectable, with its parity test, as the measured form of "a fire layer in one launch".
thread_local int g_fire_one_launch = -1;
void sq_tune_fire_one_launch(int mode) { g_fire_one_launch = mode; }
constexpr int kFireOneLaunchMaxBatch = 0;

int sq_blocked_fire_forward(const void *in, const void *packed_sq, const float *b_sq, const void *packed_e1,
                            const float *b_e1, const void *packed_e3, const float *b_e3, void *out, int N, int Cin, int H,
                            int W, int Csq, int Ce1, int Ce3, void *workspace, size_t workspace_bytes)
{
    if (!in || !packed_sq || !packed_e1 || !packed_e3 || !out) return SQ_ERR_NULL;
    if (N <= 0 || Cin <= 0 || H <= 0 || W <= 0 || Csq <= 0 || Ce1 <= 0 || Ce3 <= 0) return SQ_ERR_SHAPE;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < blocked_map_bytes(N, Csq, H, W)) return SQ_ERR_WORKSPACE;
    if (((uintptr_t)in & 15) || ((uintptr_t)out & 15) || ((uintptr_t)packed_sq & 15) || ((uintptr_t)packed_e1 & 15) ||
        ((uintptr_t)packed_e3 & 15) || Ce1 % 8 != 0)
        return SQ_ERR_UNSUPPORTED;
    if (g_fire_one_launch == 1 || (g_fire_one_launch == -1 && N <= kFireOneLaunchMaxBatch)) {
        set_stage("fire");
        const int rc1 = blocked_fire_fused(in, packed_sq, b_sq, packed_e1, b_e1, packed_e3, b_e3, out, N, Cin, H, W, Csq, Ce1, Ce3);
        set_stage("");
        if (rc1 != SQ_ERR_UNSUPPORTED) return rc1;
    }
    set_stage(kFireAlone[0]);
    int rc = blocked_conv(in, packed_sq, b_sq, workspace, N, Cin, H, W, Csq, 1, 0, 1, Csq, 0);
    if (!rc) {
        set_stage(kFireAlone[3]);
        rc = blocked_conv_pair(workspace, packed_e1, b_e1, Ce1, 0, packed_e3, b_e3, Ce3, Ce1, 3, out, N, Csq, H, W, 1, Ce1 + Ce3);
    }
    set_stage("");
    return rc;
}

int sq_blocked_maxpool(const void *in, void *out, int N, int C, int H, int W, int K, int S)
{
    if (!in || !out) return SQ_ERR_NULL;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0 || K <= 0 || S < 1 || H < K || W < K) return SQ_ERR_SHAPE;
    return blocked_maxpool(in, out, N, C, H, W, K, S);
}

int sq_blocked_avgpool_global(const void *in, float *out, int N, int C, int H, int W)
{
    if (!in || !out) return SQ_ERR_NULL;
    if (N <= 0 || C <= 0 || H <= 0 || W <= 0) return SQ_ERR_SHAPE;
    return blocked_avgpool_global(in, out, N, C, H, W);
}

// Which poolings of the reduced-precision network run inside the following squeeze launch (bit 0: pool1,
// bit 1: pool4, bit 2: pool8); -1 = the default policy.  Measured on MI355X, whole passes at batches 1 to 256,
// with the fused fire layer writing over its own input: pool1 pays at every batch (3-4 % of the pass at batch
// 64), pool4 from batch 32 on (below, its 16 dependent steps of nine loads are slower than two short launches),
// pool8 at none (its squeeze has 512 input layers: 32 dependent steps of nine loads each on few pixels; the
// pooling kernel that issues a window's nine loads at once is faster at every batch, by 0.5 % of the pass at
// batches 128 and 256).  The setter is a tuning hook, not part of the public interface.
thread_local int g_fuse_pools = -1;
void sq_tune_fuse_pools(int mask) { g_fuse_pools = mask; }

namespace {
// (Cout, Cin, K) of convolution i of the network, i = 0 (conv1) .. 25 (conv10)
void net_conv_shape(int i, int &cout, int &cin, int &k)
{
    if (i == 0) { cout = 96; cin = 3; k = 7; return; }
    if (i == 25) { cout = 1000; cin = 512; k = 1; return; }
    const int f = (i - 1) / 3, part = (i - 1) % 3;
    const FireCfg &fc = kFires[f];
    if (part == 0) { cout = fc.sq; cin = fc.cin; k = 1; }
    else { cout = fc.e; cin = fc.sq; k = part == 1 ? 1 : 3; }
}
// byte offset of convolution i's packed kernels inside the packed buffer
size_t net_packed_offset(int i)
{
    size_t off = 0;
    for (int q = 0; q < i; ++q) {
        int cout, cin, k;
        net_conv_shape(q, cout, cin, k);
        off += align_up(q == 0 ? blocked_packed_kernel7_bytes() : blocked_packed_kernel_bytes(cout, cin, k), 256);
    }
    return off;
}
}  // namespace

size_t sq_squeezenet_bf16_packed_bytes(void) { return net_packed_offset(26); }

int sq_squeezenet_bf16_pack_params(const void *const *params, void *packed, size_t packed_bytes)
{
    if (!params || !packed) return SQ_ERR_NULL;
    for (int i = 0; i < 52; ++i)
        if (!params[i]) return SQ_ERR_NULL;
    if (((uintptr_t)packed & 255) || packed_bytes < sq_squeezenet_bf16_packed_bytes()) return SQ_ERR_WORKSPACE;
    int rc = blocked_pack_kernels7(params[0], SQ_F32, packed, 96);
    if (rc) return rc;
    for (int i = 1; i < 26; ++i) {
        int cout, cin, k;
        net_conv_shape(i, cout, cin, k);
        if ((rc = blocked_pack_kernels(params[2 * i], SQ_F32, (char *)packed + net_packed_offset(i), cout, cin, k))) return rc;
    }
    return SQ_OK;
}

size_t sq_squeezenet_bf16_workspace_bytes(int N)
{
    if (N <= 0) return 0;
    const size_t n = (size_t)N;
    // two alternating maps, the squeeze map, the class means (element counts as in the fp32 network, 2 bytes each)
    return align_up(n * kBufA * 2, 256) + align_up(n * kBufB * 2, 256) + align_up(n * kBufS * 2, 256) +
           align_up(n * 1000 * 4, 256);
}

int sq_squeezenet_forward_bf16(const void *in, sq_dtype in_dtype, const void *const *params, const void *packed,
                               float *probs, int N, void *workspace, size_t workspace_bytes, float *const *taps)
{
    if (!in || !params || !packed || !probs) return SQ_ERR_NULL;
    if (N <= 0) return SQ_ERR_SHAPE;
    if (N > SQ_SQUEEZENET_BF16_MAX_BATCH) return SQ_ERR_UNSUPPORTED;   // conv1's output would pass 2^31 bytes
    if (in_dtype != SQ_F32 && in_dtype != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    for (int i = 0; i < 52; ++i)
        if (!params[i]) return SQ_ERR_NULL;
    if (taps && taps[15]) return SQ_ERR_UNSUPPORTED;
    if ((uintptr_t)packed & 255) return SQ_ERR_WORKSPACE;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < sq_squeezenet_bf16_workspace_bytes(N))
        return SQ_ERR_WORKSPACE;

    const size_t n = (size_t)N;
    char *base = (char *)workspace;
    char *bufA = base;
    char *bufB = bufA + align_up(n * kBufA * 2, 256);
    char *bufS = bufB + align_up(n * kBufB * 2, 256);
    float *means = (float *)(bufS + align_up(n * kBufS * 2, 256));
    auto B = [&](int conv) { return (const float *)params[2 * conv + 1]; };
    auto WP = [&](int conv) { return (const void *)((const char *)packed + net_packed_offset(conv)); };
    // fp32 NCHW copy of a blocked stage result for the caller
    auto tap_out = [&](int i, const void *map, int C, int H) -> int {
        if (!taps || !taps[i]) return SQ_OK;
        return blocked_unpack_map(map, taps[i], N, C, H, H);
    };

    int rc = SQ_OK;
    set_stage("conv1");
    if ((rc = blocked_conv7s2(in, in_dtype, WP(0), B(0), bufA, N, 224, 224, 96, 2, 1, 96, 0))) return rc;
    if ((rc = tap_out(0, bufA, 96, 111))) return rc;
    // Each pooled map is read by exactly one squeeze layer, so pooling runs inside that layer's launch and the
    // pooled map is never written -- unless the caller wants to see it (taps), then the two run separately
    // (same results bit for bit).
    const int fuse_pools = taps != nullptr ? 0 : g_fuse_pools >= 0 ? g_fuse_pools : (1 | (N >= 32 ? 2 : 0));
    char *cur = bufA, *nxt = bufB;
    int C = 96, H = 111, tap = 1;
    bool pool_pending = true;       // `cur` still has to be pooled (3x3, stride 2) before the next squeeze
    static const char *const kPoolSq[3] = {"pool1+fire2/sq", "pool4+fire5/sq", "pool8+fire9/sq"};
    for (int f = 0; f < 8; ++f) {
        const FireCfg &fc = kFires[f];
        const int c0 = 1 + 3 * f;
        const int which_pool = f == 0 ? 0 : f == 3 ? 1 : 2;
        // small batches: the whole fire layer in one launch (then its pooling, if any, runs on its own)
        const bool one_launch = (g_fire_one_launch == 1 || (g_fire_one_launch == -1 && N <= kFireOneLaunchMaxBatch)) &&
                                blocked_fire_fused_supported(C, fc.sq, fc.e, fc.e, pool_pending ? (H - 3) / 2 + 1 : H);
        if (pool_pending && (one_launch || !((fuse_pools >> which_pool) & 1))) {
            set_stage(f == 0 ? "pool1" : f == 3 ? "pool4" : "pool8");
            if ((rc = blocked_maxpool(cur, nxt, N, C, H, H, 3, 2))) return rc;
            H = (H - 3) / 2 + 1;
            if ((rc = tap_out(tap++, nxt, C, H))) return rc;
            { char *t = cur; cur = nxt; nxt = t; }
            pool_pending = false;
        }
        if (one_launch) {
            set_stage(kFireStages[f][3]);
            if ((rc = blocked_fire_fused(cur, WP(c0), B(c0), WP(c0 + 1), B(c0 + 1), WP(c0 + 2), B(c0 + 2), nxt, N, C, H, H, fc.sq,
                                         fc.e, fc.e)))
                return rc;
        } else {
            if (pool_pending) {
                set_stage(kPoolSq[which_pool]);
                if ((rc = blocked_pool_conv(cur, WP(c0), B(c0), bufS, N, C, H, H, fc.sq, 1, fc.sq, 0))) return rc;
                H = (H - 3) / 2 + 1;
                pool_pending = false;
                // only the squeeze reads this layer's input: the expands write over it, so that every later
                // layer finds its maps in the same buffer as without the fusion
                { char *t = cur; cur = nxt; nxt = t; }
            } else {
                set_stage(kFireStages[f][0]);
                if ((rc = blocked_conv(cur, WP(c0), B(c0), bufS, N, C, H, H, fc.sq, 1, 0, 1, fc.sq, 0))) return rc;
            }
            // both expands in one launch
            set_stage(kFireStages[f][3]);
            if ((rc = blocked_conv_pair(bufS, WP(c0 + 1), B(c0 + 1), fc.e, 0, WP(c0 + 2), B(c0 + 2), fc.e, fc.e, 3, nxt, N, fc.sq, H,
                                        H, 1, 2 * fc.e)))
                return rc;
        }
        C = 2 * fc.e;
        if ((rc = tap_out(tap++, nxt, C, H))) return rc;
        { char *t = cur; cur = nxt; nxt = t; }
        pool_pending = f == 2 || f == 6;   // pooling follows fire4 and fire8
    }
    set_stage("conv10");
    if ((rc = blocked_conv(cur, WP(25), B(25), nxt, N, 512, H, H, 1000, 1, 0, 1, 1000, 0))) return rc;
    if ((rc = tap_out(12, nxt, 1000, H))) return rc;
    set_stage("avgpool");
    if ((rc = blocked_avgpool_global(nxt, means, N, 1000, H, H))) return rc;
    if ((rc = copy_tap(taps, 13, means, n * 1000))) return rc;
    set_stage("softmax");
    if ((rc = softmax(means, probs, N, 1000))) return rc;
    set_stage("");
    return copy_tap(taps, 14, probs, n * 1000);
}

}  // extern "C"
