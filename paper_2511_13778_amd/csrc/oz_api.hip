// C ABI of the library (see include/ozdgemm.h): argument checking, workspace layout and the
// fixed, data-independent sequence of kernel launches.  Every kernel is enqueued on every call;
// the ones after the verdict read the device-resident record and return at once when they are
// not selected, so no host-device synchronisation is needed to route a call
// (paper: section "GPU-Resident Integration" and the flowchart of the GEMM decision process).
#include <cstring>
#include <new>
#include <vector>

#include "oz_internal.h"

// Workspace of oz_dgemm_static: device memory owned by the library, one copy per GPU that loads
// it, held until the process ends.  In host code this name is only a handle for
// hipGetSymbolAddress; the device address obtained there (per device, in oz_create) is what the
// kernels are given.
static __device__ __align__(256) unsigned char scratch[OZ_STATIC_SCRATCH_BYTES];

struct oz_handle {
    int device;
    int num_cu;
    void* static_ws;      // device address of `scratch` on this handle's device
    // lanes of oz_dgemm_strided_batched: streams (default priority) and the events that fork them
    // from, and join them to, the caller's stream; created once in oz_create
    hipStream_t lane[OZ_BATCH_LANES];
    hipEvent_t lane_done[OZ_BATCH_LANES];
    hipEvent_t fork;
    bool lanes_ok;
    oz_heuristic_t hm;
    // stage timing
    int prof_calls;       // calls still to be recorded
    int prof_next;        // index of the next call to record
    std::vector<hipEvent_t> events;   // (OZ_NUM_STAGES + 1) per recorded call
};

namespace {

using namespace oz;

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

bool parse_trans(char c, bool& t) {
    if (c == 'N' || c == 'n') { t = false; return true; }
    if (c == 'T' || c == 't') { t = true; return true; }
    return false;
}

bool valid_opts(const oz_opts_t& o) {
    if (o.mode < OZ_DYNAMIC || o.mode > OZ_NATIVE) return false;
    if (o.target_bits < 1 || o.target_bits > 200) return false;
    if (o.max_bits < 1 || o.max_bits > 200) return false;
    if (o.slices < 0 || o.slices > kMaxSlices) return false;
    if (o.esc_block < 0 || o.esc_block > 1024 || o.esc_block % 16 != 0) return false;
    if (o.heuristic != 0 && o.heuristic != 1) return false;
    if (o.tile_slices != 0 && o.tile_slices != 1) return false;
    return true;
}

bool emulation_slower(const oz_heuristic_t& hm, int S, int64_t m, int64_t n, int64_t k) {
    const int64_t flops = 2 * m * n * k;
    const int64_t pairs = int64_t(S) * (S + 1) / 2;
    // bytes the streaming stages move: scan 8, slicing 8 + S per operand element; per element of C the slice GEMM
    // writes and the recomposition reads 4 + (S - 1) (leading word and digits), and C is read and written
    const int64_t stream = (16 + S) * (m * k + k * n) + (2 * int64_t(S) + 22) * m * n;
    const int64_t t_emu = hm.fixed_ns + (flops / hm.int8_ops_per_ns) * pairs + stream / hm.bytes_per_ns;
    const int64_t t_f64 = flops / hm.fp64_flops_per_ns;
    return t_emu > t_f64;
}

// largest slice count a call with these options can select
int slice_cap(const oz_handle& h, const oz_opts_t& o, int64_t m, int64_t n, int64_t k) {
    if (o.mode == OZ_NATIVE) return 1;
    if (o.mode != OZ_DYNAMIC) {
        int s = o.slices > 0 ? o.slices : (o.max_bits + 1 + 7) / 8;
        return s < 1 ? 1 : (s > kMaxSlices ? kMaxSlices : s);
    }
    int s = (o.max_bits + 1 + kHeadroomBits + 7) / 8;
    if (s > kMaxSlices) s = kMaxSlices;
    // One slice count for all of C: the cost model is monotone in S, beyond this the verdict is
    // "slower".  With per-tile counts the model sees the mean pair count, so a few blocks may take any
    // count max_bits allows while the call still pays: no tighter cap than max_bits.
    if (o.heuristic && !o.tile_slices)
        while (s > 1 && emulation_slower(h.hm, s, m, n, k)) --s;
    return s;
}

bool make_problem(const oz_handle& h, const oz_opts_t& o, int64_t m, int64_t n, int64_t k, Problem& p) {
    if (m < 0 || n < 0 || k < 0) return false;
    // per-dimension limits keep every launch grid inside what the device accepts (the kernels that
    // put k or n on grid.y launch in slabs); the limit on the product keeps 2mnk and the cost
    // model's other terms inside int64
    if (m > kMaxRows || n > kMaxRows || k > kMaxK) return false;
    if (static_cast<unsigned __int128>(m) * static_cast<unsigned __int128>(n) * static_cast<unsigned __int128>(k) >
        static_cast<unsigned __int128>(kMaxMnk))
        return false;
    p.m = m; p.n = n; p.k = k;
    p.mp = round_up(m > 0 ? m : 1, kRowPad);
    p.np = round_up(n > 0 ? n : 1, kRowPad);
    p.kp = round_up(k > 0 ? k : 1, kKPad);
    p.s_cap = slice_cap(h, o, m, n, k);
    p.kblk = k_block_length(p.s_cap);
    p.nkb = int((p.kp + p.kblk - 1) / p.kblk);
    p.esc_block = o.esc_block > 0 ? o.esc_block : kDefaultEscBlock;
    p.G = int((p.k + p.esc_block - 1) / p.esc_block);
    if (p.G < 1) p.G = 1;
    p.num_cu = h.num_cu;
    p.tile_mode = (o.mode == OZ_DYNAMIC && o.tile_slices) ? 1 : 0;
    const int64_t tiles = (p.mp / kTile) * (p.np / kTile);
    p.raw_slots = int(tiles < h.num_cu ? tiles : h.num_cu);
    return true;
}

// inner length of the BF16-encoded block tables: 2G rounded up to two MFMA K-steps of 16
size_t enc_rows(const Problem& p) { return size_t((2 * p.G + 31) / 32) * 32; }

void make_layout(const Problem& p, oz_layout_t& L) {
    size_t off = 0;
    L.mp = p.mp; L.np = p.np; L.kp = p.kp; L.s_cap = p.s_cap; L.nkb = p.nkb; L.kblk = p.kblk;
    L.off_record = off; off = align_up(off + sizeof(Record));
    L.off_eA = off; off = align_up(off + size_t(p.mp) * 4);
    L.off_eB = off; off = align_up(off + size_t(p.np) * 4);
    // block tables (not part of the published layout)
    off = align_up(off + size_t(2) * p.G * p.mp * 2);
    off = align_up(off + size_t(2) * p.G * p.np * 2);
    off = align_up(off + enc_rows(p) * p.mp * 2);
    off = align_up(off + enc_rows(p) * p.np * 2);
    L.off_As = off; off = align_up(off + size_t(p.s_cap) * p.kp * p.mp);
    L.off_Bs = off; off = align_up(off + size_t(p.s_cap) * p.kp * p.np);
    L.off_T = off; off = align_up(off + size_t(p.nkb) * p.np * p.mp * 4);
    L.off_L = off; off = align_up(off + size_t(p.nkb) * (p.s_cap - 1) * p.np * p.mp);
    // raw sums of split tiles (not part of the published layout)
    off = align_up(off + size_t(p.nkb) * p.s_cap * p.raw_slots * kTile * kTile * 4);
    const size_t tiles = size_t(p.mp / kTile) * size_t(p.np / kTile);
    off = align_up(off + tiles * 4);                 // tile_span (not part of the published layout)
    L.off_tileS = off; off = align_up(off + tiles * 8);   // slice counts, then the order the tiles are dealt in
    L.total_bytes = off;
}

Workspace bind(void* base, const Problem& p, const oz_layout_t& L) {
    uint8_t* b = static_cast<uint8_t*>(base);
    Workspace w;
    w.rec = reinterpret_cast<Record*>(b + L.off_record);
    w.eA = reinterpret_cast<int32_t*>(b + L.off_eA);
    w.eB = reinterpret_cast<int32_t*>(b + L.off_eB);
    size_t offU = align_up(L.off_eB + size_t(p.np) * 4);
    size_t offV = align_up(offU + size_t(2) * p.G * p.mp * 2);
    size_t offEU = align_up(offV + size_t(2) * p.G * p.np * 2);
    size_t offEV = align_up(offEU + enc_rows(p) * p.mp * 2);
    w.U = reinterpret_cast<int16_t*>(b + offU);
    w.V = reinterpret_cast<int16_t*>(b + offV);
    w.EU = reinterpret_cast<uint16_t*>(b + offEU);
    w.EV = reinterpret_cast<uint16_t*>(b + offEV);
    w.As = reinterpret_cast<int8_t*>(b + L.off_As);
    w.Bs = reinterpret_cast<int8_t*>(b + L.off_Bs);
    w.T = reinterpret_cast<int32_t*>(b + L.off_T);
    w.L = reinterpret_cast<int8_t*>(b + L.off_L);
    const size_t off_raw = align_up(L.off_L + size_t(p.nkb) * (p.s_cap - 1) * p.np * p.mp);
    w.raw = reinterpret_cast<int32_t*>(b + off_raw);
    w.tile_span = reinterpret_cast<int32_t*>(b + align_up(off_raw + size_t(p.nkb) * p.s_cap * p.raw_slots * kTile * kTile * 4));
    w.tile_S = reinterpret_cast<int32_t*>(b + L.off_tileS);
    return w;
}

// the handle is bound to one device; kernels launch on the current one
bool on_handle_device(const oz_handle& h) {
    int dev = -1;
    return hipGetDevice(&dev) == hipSuccess && dev == h.device;
}

bool check_dims(bool ta, bool tb, int64_t m, int64_t n, int64_t k, int64_t lda, int64_t ldb, int64_t ldc) {
    const int64_t rows_a = ta ? k : m, rows_b = tb ? n : k;
    if (lda < (rows_a > 1 ? rows_a : 1)) return false;
    if (ldb < (rows_b > 1 ? rows_b : 1)) return false;
    if (ldc < (m > 1 ? m : 1)) return false;
    return true;
}

// records the event closing stage `stage` of the profiled call, if profiling is active
struct StageClock {
    oz_handle* h;
    hipStream_t st;
    hipEvent_t* ev;
    StageClock(oz_handle* hh, hipStream_t s, bool enabled = true) : h(hh), st(s), ev(nullptr) {
        if (enabled && h->prof_calls > 0 && size_t(h->prof_next + 1) * (OZ_NUM_STAGES + 1) <= h->events.size()) {
            ev = &h->events[size_t(h->prof_next) * (OZ_NUM_STAGES + 1)];
            --h->prof_calls;
            ++h->prof_next;
            (void)hipEventRecord(ev[0], st);
        }
    }
    void done(int stage) { if (ev) (void)hipEventRecord(ev[stage + 1], st); }
};

}  // namespace

extern "C" {

const char* oz_status_string(oz_status_t s) {
    switch (s) {
        case OZ_OK: return "ok";
        case OZ_ERR_ARG: return "invalid argument";
        case OZ_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case OZ_ERR_DEVICE: return "device is not gfx950 or cannot be used";
        case OZ_ERR_HIP: return "HIP runtime call failed";
    }
    return "unknown status";
}

void oz_default_opts(oz_opts_t* o) {
    if (!o) return;
    o->mode = OZ_DYNAMIC;
    o->target_bits = 53;
    o->max_bits = 200;
    o->slices = 0;
    o->esc_block = 0;
    o->heuristic = 1;
    o->tile_slices = 1;
}

oz_status_t oz_create(oz_handle_t* handle, int device) {
    if (!handle) return OZ_ERR_ARG;
    *handle = nullptr;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return OZ_ERR_DEVICE;
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return OZ_ERR_DEVICE;
    oz_handle* h = new (std::nothrow) oz_handle();
    if (!h) return OZ_ERR_ARG;
    h->device = device;
    h->num_cu = prop.multiProcessorCount;
    {
        // every GPU holds its own copy of the static workspace at its own address: resolve it with
        // the handle's device current, then put the caller's device back
        int prev = -1;
        h->static_ws = nullptr;
        bool ok = hipGetDevice(&prev) == hipSuccess && hipSetDevice(device) == hipSuccess &&
                  hipGetSymbolAddress(&h->static_ws, HIP_SYMBOL(scratch)) == hipSuccess && h->static_ws != nullptr;
        if (prev >= 0 && prev != device) ok = (hipSetDevice(prev) == hipSuccess) && ok;
        if (!ok) {
            delete h;
            return OZ_ERR_HIP;
        }
    }
    {
        // side streams for batched calls; a handle without them still works (batches then run serially)
        int prev = -1;
        h->lanes_ok = hipGetDevice(&prev) == hipSuccess && hipSetDevice(device) == hipSuccess;
        for (int l = 0; l < OZ_BATCH_LANES; ++l) { h->lane[l] = nullptr; h->lane_done[l] = nullptr; }
        h->fork = nullptr;
        if (h->lanes_ok) {
            h->lanes_ok = hipEventCreateWithFlags(&h->fork, hipEventDisableTiming) == hipSuccess;
            for (int l = 0; l < OZ_BATCH_LANES && h->lanes_ok; ++l)
                h->lanes_ok = hipStreamCreateWithFlags(&h->lane[l], hipStreamNonBlocking) == hipSuccess &&
                              hipEventCreateWithFlags(&h->lane_done[l], hipEventDisableTiming) == hipSuccess;
        }
        if (prev >= 0 && prev != device) (void)hipSetDevice(prev);
    }
    // measured on MI355X: slice GEMM 2.6-2.9 POP/s at 8192^3 (2.65 is used), native FP64 GEMM 55-75 TFLOP/s
    // between 2304^3 and 8192^3 (74, its rate where emulation competes, is used), streaming kernels about 4 TB/s, launch overhead of the ten
    // kernels of a call
    h->hm.int8_ops_per_ns = 2650000;
    h->hm.fp64_flops_per_ns = 74000;
    h->hm.bytes_per_ns = 4000;
    h->hm.fixed_ns = 60000;
    h->prof_calls = 0;
    h->prof_next = 0;
    *handle = h;
    return OZ_OK;
}

oz_status_t oz_destroy(oz_handle_t h) {
    if (!h) return OZ_ERR_ARG;
    for (hipEvent_t e : h->events) (void)hipEventDestroy(e);
    for (int l = 0; l < OZ_BATCH_LANES; ++l) {
        if (h->lane_done[l]) (void)hipEventDestroy(h->lane_done[l]);
        if (h->lane[l]) (void)hipStreamDestroy(h->lane[l]);
    }
    if (h->fork) (void)hipEventDestroy(h->fork);
    delete h;
    return OZ_OK;
}

oz_status_t oz_set_heuristic(oz_handle_t h, const oz_heuristic_t* model) {
    if (!h || !model) return OZ_ERR_ARG;
    if (model->int8_ops_per_ns <= 0 || model->fp64_flops_per_ns <= 0 || model->bytes_per_ns <= 0 ||
        model->fixed_ns < 0)
        return OZ_ERR_ARG;
    h->hm = *model;
    return OZ_OK;
}

oz_status_t oz_dgemm_layout(oz_handle_t h, char transa, char transb, int64_t m, int64_t n, int64_t k,
                            const oz_opts_t* opts, oz_layout_t* layout) {
    bool ta, tb;
    if (!h || !opts || !layout || !parse_trans(transa, ta) || !parse_trans(transb, tb)) return OZ_ERR_ARG;
    if (!valid_opts(*opts)) return OZ_ERR_ARG;
    Problem p;
    if (!make_problem(*h, *opts, m, n, k, p)) return OZ_ERR_ARG;
    make_layout(p, *layout);
    return OZ_OK;
}

size_t oz_dgemm_workspace_bytes(oz_handle_t h, char transa, char transb, int64_t m, int64_t n, int64_t k,
                                const oz_opts_t* opts) {
    oz_layout_t L;
    if (oz_dgemm_layout(h, transa, transb, m, n, k, opts, &L) != OZ_OK) return 0;
    return L.total_bytes;
}

oz_status_t oz_profile_enable(oz_handle_t h, int32_t max_calls) {
    if (!h || max_calls < 0 || max_calls > 4096) return OZ_ERR_ARG;
    const size_t need = size_t(max_calls) * (OZ_NUM_STAGES + 1);
    while (h->events.size() < need) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return OZ_ERR_HIP;
        h->events.push_back(e);
    }
    h->prof_calls = max_calls;
    h->prof_next = 0;
    return OZ_OK;
}

oz_status_t oz_profile_read(oz_handle_t h, int32_t call, float* stage_ms) {
    if (!h || !stage_ms || call < 0 || call >= h->prof_next) return OZ_ERR_ARG;
    hipEvent_t* ev = &h->events[size_t(call) * (OZ_NUM_STAGES + 1)];
    for (int s = 0; s < OZ_NUM_STAGES; ++s) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ev[s], ev[s + 1]) != hipSuccess) return OZ_ERR_HIP;
        stage_ms[s] = ms;
    }
    return OZ_OK;
}

oz_status_t oz_native_dgemm(oz_handle_t h, void* stream, char transa, char transb, int64_t m, int64_t n,
                            int64_t k, double alpha, const double* A, int64_t lda, const double* B,
                            int64_t ldb, double beta, double* C, int64_t ldc) {
    bool ta, tb;
    if (!h || !parse_trans(transa, ta) || !parse_trans(transb, tb)) return OZ_ERR_ARG;
    if (m < 0 || n < 0 || k < 0 || !check_dims(ta, tb, m, n, k, lda, ldb, ldc)) return OZ_ERR_ARG;
    if (m == 0 || n == 0) return OZ_OK;
    if (!C || (k > 0 && alpha != 0.0 && (!A || !B))) return OZ_ERR_ARG;
    if (!on_handle_device(*h)) return OZ_ERR_DEVICE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (k == 0 || alpha == 0.0) launch_scale_c(st, m, n, beta, C, ldc);
    else launch_dgemm_f64(st, nullptr, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc);
    return hipGetLastError() == hipSuccess ? OZ_OK : OZ_ERR_HIP;
}

}  // extern "C"

namespace {

oz_status_t dgemm_impl(oz_handle_t h, void* stream, char transa, char transb, int64_t m, int64_t n, int64_t k,
                       double alpha, const double* A, int64_t lda, const double* B, int64_t ldb, double beta,
                       double* C, int64_t ldc, const oz_opts_t* opts, void* workspace, size_t workspace_bytes,
                       oz_result_t* result, bool timed = true) {
    bool ta, tb;
    if (!h || !opts || !parse_trans(transa, ta) || !parse_trans(transb, tb)) return OZ_ERR_ARG;
    if (!valid_opts(*opts)) return OZ_ERR_ARG;
    Problem p;
    if (!make_problem(*h, *opts, m, n, k, p)) return OZ_ERR_ARG;
    if (!check_dims(ta, tb, m, n, k, lda, ldb, ldc)) return OZ_ERR_ARG;
    if (m == 0 || n == 0) return OZ_OK;
    if (!C) return OZ_ERR_ARG;
    if (!on_handle_device(*h)) return OZ_ERR_DEVICE;
    oz_layout_t L;
    make_layout(p, L);
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 || workspace_bytes < L.total_bytes)
        return OZ_ERR_WORKSPACE;

    if (k != 0 && alpha != 0.0 && (!A || !B)) return OZ_ERR_ARG;

    // every argument has been accepted: from here on the call only enqueues
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Workspace w = bind(workspace, p, L);
    StageClock clk(h, st, timed);
    // what the native GEMM may use for the partial products of a k split: the slice planes, the
    // aggregated products and the raw sums, none of which a call that falls back reads or writes
    void* const f64_scratch = w.As;
    const size_t f64_scratch_bytes = size_t(reinterpret_cast<uint8_t*>(w.tile_span) - reinterpret_cast<uint8_t*>(w.As));

    if (k == 0 || alpha == 0.0) {
        // BLAS convention: nothing to multiply
        launch_verdict(st, w, p, *opts, h->hm, 2, result);
        launch_scale_c(st, m, n, beta, C, ldc);
        for (int s = 0; s < OZ_NUM_STAGES; ++s) clk.done(s);
        return hipGetLastError() == hipSuccess ? OZ_OK : OZ_ERR_HIP;
    }

    // element (r, l) of op(A) (r = i) and of op(B) (r = j) at base[r*stride_r + l*stride_l]
    const int64_t a_sr = ta ? lda : 1, a_sl = ta ? 1 : lda;
    const int64_t b_sr = tb ? 1 : ldb, b_sl = tb ? ldb : 1;

    if (opts->mode == OZ_NATIVE) {
        launch_verdict(st, w, p, *opts, h->hm, 0, result);
        for (int s = 0; s <= 5; ++s) clk.done(s);
        launch_dgemm_f64(st, nullptr, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, f64_scratch, f64_scratch_bytes);
        clk.done(6);
        return hipGetLastError() == hipSuccess ? OZ_OK : OZ_ERR_HIP;
    }

    if (opts->mode == OZ_DYNAMIC && opts->heuristic) {
        // the ESC is at least 1: no input gets fewer slices than this; if even that count is slower
        // than the native GEMM by the cost model, the operands need not be scanned at all
        int s_min = (opts->target_bits + 1 + 1 + kHeadroomBits + 7) / 8;
        if (s_min > kMaxSlices) s_min = kMaxSlices;
        if (emulation_slower(h->hm, s_min, m, n, k)) {
            launch_verdict(st, w, p, *opts, h->hm, 3, result);
            for (int s = 0; s <= 5; ++s) clk.done(s);
            launch_dgemm_f64(st, nullptr, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, f64_scratch, f64_scratch_bytes);
            clk.done(6);
            return hipGetLastError() == hipSuccess ? OZ_OK : OZ_ERR_HIP;
        }
    }

    const bool guarded = opts->mode != OZ_FIXED_UNGUARDED;
    launch_init(st, w, p);
    launch_scan(st, A, a_sr, a_sl, m, p.mp, p, w.U, /*max_first=*/true, w.eA, w.rec, guarded);
    launch_scan(st, B, b_sr, b_sl, n, p.np, p, w.V, /*max_first=*/false, w.eB, w.rec, guarded);
    clk.done(0);
    if (guarded) launch_esc(st, w, p);
    clk.done(1);
    if (p.tile_mode) launch_tile_verdict(st, w, p, *opts);
    launch_verdict(st, w, p, *opts, h->hm, guarded ? 1 : 0, result);
    clk.done(2);
    launch_slice(st, A, a_sr, a_sl, m, p.mp, p, w.eA, w.As, w.rec);
    launch_slice(st, B, b_sr, b_sl, n, p.np, p, w.eB, w.Bs, w.rec);
    clk.done(3);
    launch_gemm_i8(st, w, p);
    clk.done(4);
    launch_recompose(st, w, p, alpha, beta, C, ldc);
    clk.done(5);
    if (guarded) launch_dgemm_f64(st, w.rec, ta, tb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, f64_scratch, f64_scratch_bytes);
    clk.done(6);
    return hipGetLastError() == hipSuccess ? OZ_OK : OZ_ERR_HIP;
}

}  // namespace

extern "C" {

oz_status_t oz_dgemm(oz_handle_t h, void* stream, char transa, char transb, int64_t m, int64_t n, int64_t k,
                     double alpha, const double* A, int64_t lda, const double* B, int64_t ldb, double beta,
                     double* C, int64_t ldc, const oz_opts_t* opts, void* workspace, size_t workspace_bytes,
                     oz_result_t* result) {
    return dgemm_impl(h, stream, transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, opts, workspace,
                      workspace_bytes, result);
}

// Same call with the library's static device array as the workspace: nothing is allocated, here or
// in anything this calls (kernel launches and event records only).  A problem whose workspace
// would not fit the array is refused before anything is enqueued.
oz_status_t oz_dgemm_static(oz_handle_t h, void* stream, char transa, char transb, int64_t m, int64_t n,
                            int64_t k, double alpha, const double* A, int64_t lda, const double* B, int64_t ldb,
                            double beta, double* C, int64_t ldc, const oz_opts_t* opts, oz_result_t* result) {
    if (!h) return OZ_ERR_ARG;
    return dgemm_impl(h, stream, transa, transb, m, n, k, alpha, A, lda, B, ldb, beta, C, ldc, opts, h->static_ws,
                      size_t(OZ_STATIC_SCRATCH_BYTES), result);
}

namespace {

// op in {N, T, C} of a complex operand: transposed? conjugated?
bool parse_ztrans(char c, bool& t, bool& conj) {
    conj = (c == 'C' || c == 'c');
    if (conj) { t = true; return true; }
    return parse_trans(c, t);
}

struct ZLayout {
    size_t off_ar, off_ai, off_br, off_bi, off_pr, off_pi, off_ws, total;
    size_t real_ws;
};

// planar copies of the stored A and B, the planar product, then the workspace of one real call
// (the four real products run one after the other and share it)
bool make_zlayout(oz_handle_t h, char ta_real, char tb_real, int64_t m, int64_t n, int64_t k, const oz_opts_t* opts,
                  ZLayout& z) {
    const size_t real_ws = oz_dgemm_workspace_bytes(h, ta_real, tb_real, m, n, k, opts);
    if (real_ws == 0 && m > 0 && n > 0) return false;
    size_t off = 0;
    const size_t a = align_up(size_t(m) * k * 8), b = align_up(size_t(k) * n * 8), p = align_up(size_t(m) * n * 8);
    z.off_ar = off; off += a;
    z.off_ai = off; off += a;
    z.off_br = off; off += b;
    z.off_bi = off; off += b;
    z.off_pr = off; off += p;
    z.off_pi = off; off += p;
    z.off_ws = off; off += align_up(real_ws);
    z.real_ws = real_ws;
    z.total = off;
    return true;
}

}  // namespace

size_t oz_zgemm_workspace_bytes(oz_handle_t h, char transa, char transb, int64_t m, int64_t n, int64_t k,
                                const oz_opts_t* opts) {
    bool ta, tb, ca, cb;
    if (!h || !opts || !parse_ztrans(transa, ta, ca) || !parse_ztrans(transb, tb, cb)) return 0;
    ZLayout z;
    if (!make_zlayout(h, ta ? 'T' : 'N', tb ? 'T' : 'N', m, n, k, opts, z)) return 0;
    return z.total;
}

oz_status_t oz_zgemm(oz_handle_t h, void* stream, char transa, char transb, int64_t m, int64_t n, int64_t k,
                     const double* alpha, const void* A, int64_t lda, const void* B, int64_t ldb,
                     const double* beta, void* C, int64_t ldc, const oz_opts_t* opts, void* workspace,
                     size_t workspace_bytes, oz_result_t* results) {
    bool ta, tb, ca, cb;
    if (!h || !opts || !alpha || !beta || !parse_ztrans(transa, ta, ca) || !parse_ztrans(transb, tb, cb)) return OZ_ERR_ARG;
    if (!valid_opts(*opts)) return OZ_ERR_ARG;
    if (m < 0 || n < 0 || k < 0 || !check_dims(ta, tb, m, n, k, lda, ldb, ldc)) return OZ_ERR_ARG;
    if (m == 0 || n == 0) return OZ_OK;
    if (!C || (k > 0 && (!A || !B))) return OZ_ERR_ARG;
    const char tra = ta ? 'T' : 'N', trb = tb ? 'T' : 'N';
    ZLayout z;
    if (!make_zlayout(h, tra, trb, m, n, k, opts, z)) return OZ_ERR_ARG;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 || workspace_bytes < z.total)
        return OZ_ERR_WORKSPACE;
    if (!on_handle_device(*h)) return OZ_ERR_DEVICE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t* w = static_cast<uint8_t*>(workspace);
    double* Ar = reinterpret_cast<double*>(w + z.off_ar);
    double* Ai = reinterpret_cast<double*>(w + z.off_ai);
    double* Br = reinterpret_cast<double*>(w + z.off_br);
    double* Bi = reinterpret_cast<double*>(w + z.off_bi);
    double* Pr = reinterpret_cast<double*>(w + z.off_pr);
    double* Pi = reinterpret_cast<double*>(w + z.off_pi);
    // planar parts keep the stored shape (rows x cols of the stored matrix), leading dimension = rows
    const int64_t a_rows = ta ? k : m, a_cols = ta ? m : k, b_rows = tb ? n : k, b_cols = tb ? k : n;
    launch_zsplit(st, A, lda, a_rows, a_cols, Ar, Ai, ca);
    launch_zsplit(st, B, ldb, b_rows, b_cols, Br, Bi, cb);
    const int64_t pa = a_rows > 1 ? a_rows : 1, pb = b_rows > 1 ? b_rows : 1, pm = m;
    struct Call { const double* a; const double* b; double alpha, beta; double* c; };
    const Call calls[4] = {{Ar, Br, 1.0, 0.0, Pr}, {Ai, Bi, -1.0, 1.0, Pr}, {Ar, Bi, 1.0, 0.0, Pi}, {Ai, Br, 1.0, 1.0, Pi}};
    for (int c = 0; c < 4; ++c) {
        const oz_status_t s = dgemm_impl(h, stream, tra, trb, m, n, k, calls[c].alpha, calls[c].a, pa, calls[c].b, pb,
                                         calls[c].beta, calls[c].c, pm, opts, w + z.off_ws, z.real_ws,
                                         results ? results + c : nullptr);
        if (s != OZ_OK) return s;
    }
    launch_zcombine(st, Pr, Pi, m, n, alpha[0], alpha[1], beta[0], beta[1], C, ldc);
    return hipGetLastError() == hipSuccess ? OZ_OK : OZ_ERR_HIP;
}

oz_status_t oz_dgemm_strided_batched(oz_handle_t h, void* stream, char transa, char transb, int64_t m,
                                     int64_t n, int64_t k, double alpha, const double* A, int64_t lda,
                                     int64_t stride_a, const double* B, int64_t ldb, int64_t stride_b,
                                     double beta, double* C, int64_t ldc, int64_t stride_c,
                                     int64_t batch_count, const oz_opts_t* opts, void* workspace,
                                     size_t workspace_bytes, oz_result_t* results) {
    if (batch_count < 0 || stride_a < 0 || stride_b < 0 || stride_c < 0) return OZ_ERR_ARG;
    if (batch_count > 1 && m > 0 && n > 0 && stride_c < ldc * (n - 1) + m) return OZ_ERR_ARG;   // C blocks overlap
    // validate everything once, before the first problem is enqueued
    bool ta, tb;
    if (!h || !opts || !parse_trans(transa, ta) || !parse_trans(transb, tb) || !valid_opts(*opts)) return OZ_ERR_ARG;
    if (!check_dims(ta, tb, m, n, k, lda, ldb, ldc)) return OZ_ERR_ARG;
    if (batch_count > 0 && oz_dgemm_workspace_bytes(h, transa, transb, m, n, k, opts) > workspace_bytes)
        return OZ_ERR_WORKSPACE;
    if (batch_count == 0 || m == 0 || n == 0) return OZ_OK;
    const size_t need = align_up(oz_dgemm_workspace_bytes(h, transa, transb, m, n, k, opts));
    // Lanes: as many problems in flight as the workspace has room for (one slice of `need` bytes each),
    // at most OZ_BATCH_LANES.  One lane = the caller's stream alone, problems one after the other.
    int lanes = 1;
    if (h->lanes_ok && need > 0) {
        const size_t fit = workspace_bytes / need;
        lanes = int(fit < size_t(OZ_BATCH_LANES) ? fit : size_t(OZ_BATCH_LANES));
        if (int64_t(lanes) > batch_count) lanes = int(batch_count);
        if (lanes < 1) lanes = 1;
    }
    hipStream_t user = static_cast<hipStream_t>(stream);
    if (lanes > 1) {
        if (!on_handle_device(*h)) return OZ_ERR_DEVICE;
        if (hipEventRecord(h->fork, user) != hipSuccess) return OZ_ERR_HIP;
        for (int l = 0; l < lanes; ++l)
            if (hipStreamWaitEvent(h->lane[l], h->fork, 0) != hipSuccess) return OZ_ERR_HIP;
    }
    oz_status_t status = OZ_OK;
    for (int64_t b = 0; b < batch_count && status == OZ_OK; ++b) {
        const int l = int(b % lanes);
        status = dgemm_impl(h, lanes > 1 ? h->lane[l] : user, transa, transb, m, n, k, alpha, A ? A + b * stride_a : A,
                            lda, B ? B + b * stride_b : B, ldb, beta, C ? C + b * stride_c : C, ldc, opts,
                            static_cast<uint8_t*>(workspace) + size_t(l) * need, need, results ? results + b : nullptr,
                            /*timed=*/lanes == 1);
    }
    if (lanes > 1) {
        // always join, also after an error: the caller's stream must not run ahead of what was enqueued
        for (int l = 0; l < lanes; ++l) {
            if (hipEventRecord(h->lane_done[l], h->lane[l]) != hipSuccess) status = status == OZ_OK ? OZ_ERR_HIP : status;
            if (hipStreamWaitEvent(user, h->lane_done[l], 0) != hipSuccess) status = status == OZ_OK ? OZ_ERR_HIP : status;
        }
    }
    return status;
}

}  // extern "C"
