// C ABI of libfpdt.so: argument validation, workspace planning and the host-side chunk
// schedule with its offload pipeline (Sec. 4.1 forward order, Sec. 4.2 backward order and
// double buffering).  All arithmetic lives in the kernels; this file only decides which
// chunk pair runs when, where its operands live, and which copies overlap which kernels.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/fpdt.h"
#include "fpdt_internal.h"

using namespace fpdt;

namespace {

thread_local std::string g_err;
thread_local uint64_t g_h2d_bytes = 0, g_d2h_bytes = 0;

int fail(int code, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

#define HIP_TRY(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail(FPDT_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_),  \
                        __FILE__, __LINE__);                                                  \
    } while (0)

constexpr unsigned KNOWN_FLAGS = FPDT_KV_ON_HOST | FPDT_ACT_ON_HOST | FPDT_BWD_KV_OUTER | FPDT_BWD_Q_OUTER |
                               FPDT_PAIRWISE | FPDT_BWD_STORE_DS;

struct Problem {
    int64_t S, C, u;
    int Hq, Hkv, D, dtype;
    unsigned flags;
    float scale;
    bool bf16() const { return dtype == FPDT_DTYPE_BF16; }
    size_t esize() const { return bf16() ? 2 : 4; }
    bool kv_host() const { return flags & FPDT_KV_ON_HOST; }
    bool act_host() const { return flags & FPDT_ACT_ON_HOST; }
    bool store_ds() const { return flags & FPDT_BWD_STORE_DS; }
    bool fused() const { return bf16() && !(flags & (FPDT_KV_ON_HOST | FPDT_ACT_ON_HOST | FPDT_PAIRWISE | FPDT_BWD_STORE_DS)); }
    bool q_outer() const
    {
        if (flags & FPDT_BWD_Q_OUTER) return true;
        if (flags & FPDT_BWD_KV_OUTER) return false;
        return act_host();
    }
    size_t q_chunk_bytes() const { return (size_t)C * Hq * D * esize(); }
    size_t kv_chunk_bytes() const { return (size_t)C * Hkv * D * esize(); }
    // Block-sparse variant (Sec. 5.5): u x u bytes, row = query chunk, column = key chunk; empty =
    // dense.  The diagonal is always set (checked on entry).
    std::vector<unsigned char> mask;
    bool on(int64_t m, int64_t i) const { return mask.empty() || mask[(size_t)(m * u + i)] != 0; }
    int64_t first_key_chunk(int64_t m) const { int64_t i = 0; while (!on(m, i)) ++i; return i; }
    int64_t last_query_chunk(int64_t j) const { int64_t i = u - 1; while (!on(i, j)) --i; return i; }
};

// Copy and check a caller's chunk mask (host memory, read before the entry point returns).
int take_mask(Problem& p, const unsigned char* chunk_mask)
{
    if (!chunk_mask) return fail(FPDT_ERR_INVALID_ARG, "NULL chunk mask");
    p.mask.assign(chunk_mask, chunk_mask + (size_t)(p.u * p.u));
    for (int64_t m = 0; m < p.u; ++m)
        if (!p.mask[(size_t)(m * p.u + m)])
            return fail(FPDT_ERR_INVALID_ARG, "chunk mask drops the diagonal pair (%lld, %lld): its query rows would have no key", (long long)m, (long long)m);
    return FPDT_OK;
}

// Scalar validation: touches no GPU.
int validate_scalars(Problem& p, int64_t S, int64_t chunk, int Hq, int Hkv, int D, float scale,
                     int dtype, unsigned flags)
{
    if (S <= 0 || chunk <= 0) return fail(FPDT_ERR_INVALID_ARG, "S and chunk must be positive (S=%lld chunk=%lld)", (long long)S, (long long)chunk);
    if (S % chunk != 0) return fail(FPDT_ERR_INVALID_ARG, "S=%lld is not a multiple of chunk=%lld", (long long)S, (long long)chunk);
    if (Hq <= 0 || Hkv <= 0 || Hq % Hkv != 0) return fail(FPDT_ERR_INVALID_ARG, "Hq=%d must be a positive multiple of Hkv=%d", Hq, Hkv);
    if (!(scale > 0.f) || !std::isfinite(scale)) return fail(FPDT_ERR_INVALID_ARG, "scale must be finite and > 0");
    if (dtype != FPDT_DTYPE_F32 && dtype != FPDT_DTYPE_BF16) return fail(FPDT_ERR_INVALID_ARG, "unknown dtype %d", dtype);
    if (flags & ~KNOWN_FLAGS) return fail(FPDT_ERR_INVALID_ARG, "unknown flag bits 0x%x", flags & ~KNOWN_FLAGS);
    if ((flags & FPDT_BWD_KV_OUTER) && (flags & FPDT_BWD_Q_OUTER)) return fail(FPDT_ERR_INVALID_ARG, "both loop-order flags set");
    if (D != 64 && D != 80 && D != 128) return fail(FPDT_ERR_UNSUPPORTED, "head dim %d not in {64, 80, 128}", D);
    if (dtype == FPDT_DTYPE_BF16 && chunk % FPDT_CHUNK_MULTIPLE != 0) return fail(FPDT_ERR_UNSUPPORTED, "bf16 chunk=%lld is not a multiple of %d", (long long)chunk, (int)FPDT_CHUNK_MULTIPLE);
    if (dtype == FPDT_DTYPE_F32 && (flags & (FPDT_KV_ON_HOST | FPDT_ACT_ON_HOST))) return fail(FPDT_ERR_UNSUPPORTED, "fp32 path has no host offload");
    if (dtype == FPDT_DTYPE_F32 && (flags & FPDT_BWD_STORE_DS)) return fail(FPDT_ERR_UNSUPPORTED, "fp32 path has no stored-dS backward");
    if ((flags & FPDT_BWD_STORE_DS) && (double)chunk * (double)chunk * Hq / 1024.0 >= 2147483648.0)
        return fail(FPDT_ERR_UNSUPPORTED, "stored-dS backward: chunk=%lld with %d heads has too many dS tiles (chunk^2 * Hq must stay below 2^41)", (long long)chunk, Hq);
    if ((flags & FPDT_ACT_ON_HOST) && (flags & FPDT_BWD_KV_OUTER)) return fail(FPDT_ERR_UNSUPPORTED, "FPDT_ACT_ON_HOST needs the Q-outer backward order");
    if (S > (int64_t)1 << 30 || (int64_t)Hq * (S / 32 + 1) > (int64_t)1 << 30) return fail(FPDT_ERR_UNSUPPORTED, "S=%lld beyond launch limits", (long long)S);
    p.S = S; p.C = chunk; p.u = S / chunk; p.Hq = Hq; p.Hkv = Hkv; p.D = D; p.dtype = dtype;
    p.flags = flags; p.scale = scale;
    return FPDT_OK;
}

// ---- workspace planning: the same routine sizes (base == nullptr) and carves ----
struct Bump {
    char* base;
    size_t off = 0;
    explicit Bump(void* b) : base(static_cast<char*>(b)) {}
    template <typename T = void>
    T* take(size_t bytes)
    {
        off = (off + 255) & ~(size_t)255;
        T* r = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += bytes;
        return r;
    }
};

struct FwdPlan {
    void* Knat = nullptr; void* Vtr = nullptr;
    char* kv_raw[2] = {nullptr, nullptr};
    float* st_acc = nullptr; float* st_ml = nullptr;
    char* q_buf[2] = {nullptr, nullptr};
    char* o_buf[2] = {nullptr, nullptr};
    float* lse_buf[2] = {nullptr, nullptr};
    size_t total = 0;
};

FwdPlan plan_fwd(const Problem& p, void* ws)
{
    FwdPlan f;
    Bump b(ws);
    if (!p.bf16()) {
        f.st_acc = b.take<float>((size_t)p.C * p.Hq * p.D * 4);
        f.st_ml = b.take<float>((size_t)p.C * p.Hq * 2 * 4);
    } else if (p.fused()) {
        f.Knat = b.take((size_t)(p.S / 32) * p.Hkv * nat_block_bytes(p.D));
        f.Vtr = b.take((size_t)(p.S / 32) * p.Hkv * tr_block_bytes(p.D));
    } else {
        f.Knat = b.take((size_t)(p.C / 32) * p.Hkv * nat_block_bytes(p.D));
        f.Vtr = b.take((size_t)(p.C / 32) * p.Hkv * tr_block_bytes(p.D));
        f.st_acc = b.take<float>(fwd_state_acc_bytes(p.C, p.Hq, p.D));
        f.st_ml = b.take<float>(fwd_state_ml_bytes(p.C, p.Hq, p.D));
        if (p.kv_host())
            for (int i = 0; i < 2; ++i) f.kv_raw[i] = b.take<char>(2 * p.kv_chunk_bytes());
        if (p.act_host())
            for (int i = 0; i < 2; ++i) {
                f.q_buf[i] = b.take<char>(p.q_chunk_bytes());
                f.o_buf[i] = b.take<char>(p.q_chunk_bytes());
                f.lse_buf[i] = b.take<float>((size_t)p.Hq * p.C * 4);
            }
    }
    f.total = (b.off + 255) & ~(size_t)255;
    return f;
}

struct BwdPlan {
    float* Delta = nullptr;  // [Hq, S] (resident activations) or 2 x [Hq, C] (streamed)
    float* delta_buf[2] = {nullptr, nullptr};
    void *Qnat = nullptr, *dOnat = nullptr;
    void *Knat = nullptr, *Vnat = nullptr;
    float *acc_dq = nullptr, *acc_dk = nullptr, *acc_dv = nullptr;
    char* kv_raw[2] = {nullptr, nullptr};
    char* dkv_out[2] = {nullptr, nullptr};
    char* act_raw[2] = {nullptr, nullptr};  // [Q | dO | O] chunk
    float* lse_buf[2] = {nullptr, nullptr};
    char* dq_out[2] = {nullptr, nullptr};
    void* ds_frag = nullptr;  // stored-dS backward: the dS tiles of one chunk pair
    float* stat2 = nullptr;   // row statistics of the packed query rows, as the dK/dV kernel reads them
    size_t total = 0;
};

BwdPlan plan_bwd(const Problem& p, void* ws)
{
    BwdPlan f;
    Bump b(ws);
    if (!p.bf16()) {
        f.Delta = b.take<float>((size_t)p.Hq * p.S * 4);
    } else {
        const int64_t rows = p.fused() ? p.S : p.C;  // rows covered by the packed buffers
        // NAT fragments only: the backward kernels read the row-contracted operands (Q^T, dO^T,
        // K^T) out of the NAT blocks in LDS with transposing loads
        f.Qnat = b.take((size_t)(rows / 32) * p.Hq * nat_block_bytes(p.D));
        f.dOnat = b.take((size_t)(rows / 32) * p.Hq * nat_block_bytes(p.D));
        f.Knat = b.take((size_t)(rows / 32) * p.Hkv * nat_block_bytes(p.D));
        f.Vnat = b.take((size_t)(rows / 32) * p.Hkv * nat_block_bytes(p.D));
        if (!p.act_host()) f.Delta = b.take<float>((size_t)p.Hq * p.S * 4);
        f.stat2 = b.take<float>((size_t)(rows / 32) * p.Hq * 64 * 4);
        if (!p.fused()) {
            // accumulators: the side that the outer loop holds fixed needs one chunk, the
            // other side one slot per chunk of the sequence
            const bool qo = p.q_outer();
            f.acc_dq = b.take<float>(bwd_acc_dq_bytes(qo ? p.C : p.S, p.Hq, p.D));
            f.acc_dk = b.take<float>(bwd_acc_dkv_bytes(qo ? p.S : p.C, p.Hkv, p.D));
            f.acc_dv = b.take<float>(bwd_acc_dkv_bytes(qo ? p.S : p.C, p.Hkv, p.D));
            if (p.store_ds()) f.ds_frag = b.take(bwd_ds_bytes(p.C, p.C, p.Hq));
            if (p.kv_host())
                for (int i = 0; i < 2; ++i) {
                    f.kv_raw[i] = b.take<char>(2 * p.kv_chunk_bytes());
                    f.dkv_out[i] = b.take<char>(2 * p.kv_chunk_bytes());
                }
            if (p.act_host())
                for (int i = 0; i < 2; ++i) {
                    f.act_raw[i] = b.take<char>(3 * p.q_chunk_bytes());
                    f.lse_buf[i] = b.take<float>((size_t)p.Hq * p.C * 4);
                    f.delta_buf[i] = b.take<float>((size_t)p.Hq * p.C * 4);
                    f.dq_out[i] = b.take<char>(p.q_chunk_bytes());
                }
        }
    }
    f.total = (b.off + 255) & ~(size_t)255;
    return f;
}

// ---- per-device side streams and events for the offload pipeline ----
enum Ev {
    EV_FORK, EV_JOIN_H2D, EV_JOIN_D2H,
    EV_KV_READY0, EV_KV_READY1, EV_KV_FREE0, EV_KV_FREE1,
    EV_ACT_READY0, EV_ACT_READY1, EV_ACT_FREE0, EV_ACT_FREE1,
    EV_OUT_DONE0, EV_OUT_DONE1, EV_OUT_COPIED0, EV_OUT_COPIED1,
    EV_DKV_DONE0, EV_DKV_DONE1, EV_DKV_COPIED0, EV_DKV_COPIED1,
    EV_COUNT
};

struct DeviceCtx {
    bool ready = false;
    hipStream_t h2d = nullptr, d2h = nullptr;
    hipEvent_t ev[EV_COUNT] = {};
    // event-ordering checks (fpdt_debug_configure): a pinned / device buffer pair whose copy is
    // queued in front of every staged copy to hold it back
    void* delay_host = nullptr;
    void* delay_dev = nullptr;
};
unsigned g_debug = 0;
constexpr size_t DELAY_BYTES = (size_t)48 << 20;
std::mutex g_mu;  // serialises enqueueing calls that use the shared side streams
DeviceCtx g_ctx[64];

// ---- workspace of the entry point that allocates nothing (fpdt_attn_fwd_noalloc) ----
// A file-scope device array stands in for the caller's workspace.  Every GPU the library runs
// on holds its own copy at its own address until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress: the device address is looked up once per
// device, with that device current, and only that address is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[FPDT_NOALLOC_SCRATCH_BYTES];
void* g_scratch_ptr[64] = {};
thread_local bool g_no_alloc_call = false;  // set while fpdt_attn_fwd_noalloc runs: no event creation

int scratch_for_current_device(void** out)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return fail(FPDT_ERR_HIP, "device index %d out of range", dev);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr || reinterpret_cast<uintptr_t>(ptr) % 256 != 0)
            return fail(FPDT_ERR_HIP, "static scratch array has no usable device address");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return FPDT_OK;
}

int get_ctx(DeviceCtx** out)
{
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return fail(FPDT_ERR_HIP, "device index %d out of range", dev);
    DeviceCtx& c = g_ctx[dev];
    if (!c.ready) {
        // default priority on purpose: work on streams of unequal priority is avoided; a call
        // that fails half way keeps what it made, and the next call makes only the rest
        if (!c.h2d) HIP_TRY(hipStreamCreateWithFlags(&c.h2d, hipStreamNonBlocking));
        if (!c.d2h) HIP_TRY(hipStreamCreateWithFlags(&c.d2h, hipStreamNonBlocking));
        for (int i = 0; i < EV_COUNT; ++i)
            if (!c.ev[i]) HIP_TRY(hipEventCreateWithFlags(&c.ev[i], hipEventDisableTiming));
        c.ready = true;
    }
    *out = &c;
    return FPDT_OK;
}

// Event bookkeeping of one call.  The schedules wait for "buffer free" / "copied out" events
// before they reuse a staging buffer; the first use of a buffer in a call has no such event yet
// (every buffer is free when a call starts: the call's fork orders it behind the stream's
// earlier work), and waiting there for the event's last record, which belongs to an EARLIER call,
// is not only pointless: under stream capture it is an error (a dependency on uncaptured work).
// So a wait is issued only for events this call has recorded.
struct CallEvents {
    DeviceCtx* c = nullptr;
    uint32_t seen = 0;
    static_assert(EV_COUNT <= 32, "one bit per event");
    int record(int e, hipStream_t s)
    {
        HIP_TRY(hipEventRecord(c->ev[e], s));
        seen |= 1u << e;
        return FPDT_OK;
    }
    int wait(hipStream_t s, int e)
    {
        if (!(seen & (1u << e))) return FPDT_OK;
        HIP_TRY(hipStreamWaitEvent(s, c->ev[e], 0));
        return FPDT_OK;
    }
};

// ---- pointer checks (host side, before any launch) ----
int check_ptr(const void* ptr, size_t bytes, bool want_host, const char* name)
{
    if (!ptr) return fail(FPDT_ERR_INVALID_ARG, "%s is NULL", name);
    hipPointerAttribute_t at;
    hipError_t e = hipPointerGetAttributes(&at, ptr);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(FPDT_ERR_INVALID_ARG, "%s is not %s memory known to HIP", name, want_host ? "pinned host" : "device");
    }
    if (want_host && at.type != hipMemoryTypeHost) return fail(FPDT_ERR_INVALID_ARG, "%s must be pinned host memory", name);
    if (!want_host && at.type != hipMemoryTypeDevice) return fail(FPDT_ERR_INVALID_ARG, "%s must be device memory", name);
    if (!want_host) {
        void* base = nullptr;
        size_t size = 0;
        if (hipMemGetAddressRange((hipDeviceptr_t*)&base, &size, (hipDeviceptr_t)ptr) == hipSuccess) {
            const char* end = static_cast<const char*>(base) + size;
            if (static_cast<const char*>(ptr) + bytes > end)
                return fail(FPDT_ERR_INVALID_ARG, "%s: %zu bytes run past the end of its allocation", name, bytes);
        } else {
            (void)hipGetLastError();
        }
    }
    if (reinterpret_cast<uintptr_t>(ptr) % 16 != 0) return fail(FPDT_ERR_INVALID_ARG, "%s must be 16-byte aligned", name);
    return FPDT_OK;
}

int check_workspace(void* ws, size_t have, size_t need)
{
    if (need == 0) return FPDT_OK;
    if (!ws) return fail(FPDT_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", need);
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return fail(FPDT_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    if (have < need) return fail(FPDT_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", have, need);
    int rc = check_ptr(ws, need, false, "workspace");
    if (rc != FPDT_OK) return fail(FPDT_ERR_WORKSPACE, "%s", g_err.c_str());
    return FPDT_OK;
}

int launch_status(const char* what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FPDT_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return FPDT_OK;
}

// ---- optional per-kernel timing (benchmarks): HIP events around every launch ----
struct ProfRec { int kind; hipEvent_t a, b; };
std::atomic<bool> g_prof_on{false};
std::vector<ProfRec> g_prof;
std::mutex g_prof_mu;

struct ProfScope {
    hipStream_t st;
    ProfRec r{};
    bool live = false;
    ProfScope(int kind, hipStream_t s) : st(s)
    {
        if (!g_prof_on.load(std::memory_order_relaxed) || g_no_alloc_call) return;
        if (hipEventCreate(&r.a) != hipSuccess) return;
        if (hipEventCreate(&r.b) != hipSuccess) {
            (void)hipEventDestroy(r.a);
            return;
        }
        r.kind = kind;
        live = hipEventRecord(r.a, st) == hipSuccess;
        if (!live) {
            (void)hipEventDestroy(r.a);
            (void)hipEventDestroy(r.b);
        }
    }
    ~ProfScope()
    {
        if (!live) return;
        (void)hipEventRecord(r.b, st);
        std::lock_guard<std::mutex> lk(g_prof_mu);
        g_prof.push_back(r);
    }
};
#define PROF(kind, st) ProfScope prof_scope_##__LINE__(kind, st)

// H2D / D2H helpers that keep the link-byte counters.
#define TRY(expr)                       \
    do {                                \
        int rc_ = (expr);               \
        if (rc_ != FPDT_OK) return rc_; \
    } while (0)

// With FPDT_DEBUG_DELAY_COPIES every staged copy is held back by a large dummy copy on the same
// stream; with FPDT_DEBUG_POISON_STAGING the destination of a host-to-device copy is first
// filled with 0xFF bytes (bf16 / fp32 NaNs).  A consumer that does not wait for the copy's
// event then reads NaNs, and a producer that does not wait for a buffer's release is
// overwritten late: both show up as a mismatch against the resident run.
int debug_hold_back(bool to_device, void* dst, size_t bytes, hipStream_t st)
{
    if (!g_debug) return FPDT_OK;
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    DeviceCtx& c = g_ctx[dev];
    if ((g_debug & FPDT_DEBUG_DELAY_COPIES) && c.delay_host)
        HIP_TRY(hipMemcpyAsync(to_device ? c.delay_dev : c.delay_host, to_device ? c.delay_host : c.delay_dev,
                               DELAY_BYTES, to_device ? hipMemcpyHostToDevice : hipMemcpyDeviceToHost, st));
    if ((g_debug & FPDT_DEBUG_POISON_STAGING) && to_device) launch_fill_bytes(dst, bytes, 0xFF, st);
    return FPDT_OK;
}

int copy_h2d(void* dst, const void* src, size_t bytes, hipStream_t st)
{
    TRY(debug_hold_back(true, dst, bytes, st));
    PROF(FPDT_PROF_H2D, st);
    HIP_TRY(hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, st));
    g_h2d_bytes += bytes;
    return FPDT_OK;
}
int copy_d2h(void* dst, const void* src, size_t bytes, hipStream_t st)
{
    TRY(debug_hold_back(false, nullptr, 0, st));
    PROF(FPDT_PROF_D2H, st);
    HIP_TRY(hipMemcpyAsync(dst, src, bytes, hipMemcpyDeviceToHost, st));
    g_d2h_bytes += bytes;
    return FPDT_OK;
}

// =========================================================================================
// forward
// =========================================================================================
int fwd_f32(const Problem& p, const float* Q, const float* K, const float* V, float* O, float* LSE,
            const FwdPlan& f, hipStream_t st)
{
    for (int64_t m = 0; m < p.u; ++m)
        for (int64_t i = 0; i <= m; ++i) {
            if (!p.on(m, i)) continue;
            F32FwdArgs a;
            a.Q = Q + (size_t)m * p.C * p.Hq * p.D;
            a.K = K + (size_t)i * p.C * p.Hkv * p.D;
            a.V = V + (size_t)i * p.C * p.Hkv * p.D;
            a.O = O + (size_t)m * p.C * p.Hq * p.D;
            a.LSE = LSE + m * p.C;
            a.lse_stride = p.S;
            a.st_acc = f.st_acc; a.st_ml = f.st_ml;
            a.q_pos0 = m * p.C; a.k_pos0 = i * p.C; a.n_q = p.C; a.n_k = p.C;
            a.Hq = p.Hq; a.Hkv = p.Hkv; a.D = p.D; a.scale = p.scale;
            a.flags = (i == p.first_key_chunk(m) ? SWEEP_INIT : 0) | (i == m ? SWEEP_FINAL : 0);
            launch_f32_fwd_pair(a, st);
        }
    return launch_status("fp32 forward");
}

int fwd_bf16_fused(const Problem& p, const void* Q, const void* K, const void* V, void* O, float* LSE,
                   const FwdPlan& f, hipStream_t st)
{
    launch_pack(K, p.S, p.Hkv, p.D, f.Knat, nullptr, p.S / 32, st);
    launch_pack(V, p.S, p.Hkv, p.D, nullptr, f.Vtr, p.S / 32, st);
    FwdArgs a;
    a.Q = Q; a.Knat = f.Knat; a.Vtr = f.Vtr; a.kv_head_stride_blocks = p.S / 32;
    a.O = O; a.LSE = LSE; a.lse_stride = p.S; a.st_acc = nullptr; a.st_ml = nullptr;
    a.q_pos0 = 0; a.k_pos0 = 0; a.n_q = p.S; a.n_keys = p.S;
    a.Hq = p.Hq; a.Hkv = p.Hkv; a.D = p.D; a.scale = p.scale;
    a.flags = SWEEP_INIT | SWEEP_FINAL;
    { PROF(FPDT_PROF_FWD, st); launch_fwd_sweep(a, st); }
    return launch_status("bf16 forward");
}

// Pair-by-pair forward; K/V chunks (and optionally Q/O/LSE chunks) stream through double
// buffers on the side streams while the previous pair computes.
int fwd_bf16_pairs(const Problem& p, const char* Q, const char* K, const char* V, char* O, float* LSE,
                   const FwdPlan& f, hipStream_t st)
{
    const bool kvh = p.kv_host(), acth = p.act_host();
    DeviceCtx* c = nullptr;
    CallEvents ev;
    if (kvh || acth) {
        TRY(get_ctx(&c));
        ev.c = c;
        TRY(ev.record(EV_FORK, st));
        TRY(ev.wait(c->h2d, EV_FORK));
        TRY(ev.wait(c->d2h, EV_FORK));
    }
    const size_t kvb = p.kv_chunk_bytes(), qb = p.q_chunk_bytes();

    // the K/V fetch sequence is the pair sequence
    std::vector<int64_t> kv_seq;
    for (int64_t m = 0; m < p.u; ++m)
        for (int64_t i = 0; i <= m; ++i)
            if (p.on(m, i)) kv_seq.push_back(i);
    auto fetch_kv = [&](size_t t) -> int {
        const int b = (int)(t & 1);
        TRY(ev.wait(c->h2d, EV_KV_FREE0 + b));
        TRY(copy_h2d(f.kv_raw[b], K + (size_t)kv_seq[t] * kvb, kvb, c->h2d));
        TRY(copy_h2d(f.kv_raw[b] + kvb, V + (size_t)kv_seq[t] * kvb, kvb, c->h2d));
        TRY(ev.record(EV_KV_READY0 + b, c->h2d));
        return FPDT_OK;
    };
    auto fetch_q = [&](int64_t m) -> int {
        const int b = (int)(m & 1);
        TRY(ev.wait(c->h2d, EV_ACT_FREE0 + b));
        TRY(copy_h2d(f.q_buf[b], Q + (size_t)m * qb, qb, c->h2d));
        TRY(ev.record(EV_ACT_READY0 + b, c->h2d));
        return FPDT_OK;
    };

    if (acth) TRY(fetch_q(0));
    if (kvh) TRY(fetch_kv(0));
    size_t t = 0;
    for (int64_t m = 0; m < p.u; ++m) {
        const int qbuf = (int)(m & 1);
        const char* Qm = Q + (size_t)m * qb;
        char* Om = O + (size_t)m * qb;
        float* LSEm = LSE + m * p.C;
        int64_t lse_stride = p.S;
        if (acth) {
            if (m + 1 < p.u) TRY(fetch_q(m + 1));
            TRY(ev.wait(st, EV_ACT_READY0 + qbuf));
            Qm = f.q_buf[qbuf];
            Om = f.o_buf[qbuf];
            LSEm = f.lse_buf[qbuf];
            lse_stride = p.C;
        }
        for (int64_t i = 0; i <= m; ++i) {
            if (!p.on(m, i)) continue;  // neither fetched nor computed
            const char* Ki = K + (size_t)i * kvb;
            const char* Vi = V + (size_t)i * kvb;
            if (kvh) {
                const int b = (int)(t & 1);
                if (t + 1 < kv_seq.size()) TRY(fetch_kv(t + 1));
                TRY(ev.wait(st, EV_KV_READY0 + b));
                Ki = f.kv_raw[b];
                Vi = f.kv_raw[b] + kvb;
            }
            launch_pack(Ki, p.C, p.Hkv, p.D, f.Knat, nullptr, p.C / 32, st);
            launch_pack(Vi, p.C, p.Hkv, p.D, nullptr, f.Vtr, p.C / 32, st);
            if (kvh) TRY(ev.record(EV_KV_FREE0 + (int)(t & 1), st));
            if (acth && i == m)  // the finalising sweep overwrites the staging O / LSE chunk
                TRY(ev.wait(st, EV_OUT_COPIED0 + qbuf));
            FwdArgs a;
            a.Q = Qm; a.Knat = f.Knat; a.Vtr = f.Vtr; a.kv_head_stride_blocks = p.C / 32;
            a.O = Om; a.LSE = LSEm; a.lse_stride = lse_stride;
            a.st_acc = f.st_acc; a.st_ml = f.st_ml;
            a.q_pos0 = m * p.C; a.k_pos0 = i * p.C; a.n_q = p.C; a.n_keys = p.C;
            a.Hq = p.Hq; a.Hkv = p.Hkv; a.D = p.D; a.scale = p.scale;
            a.flags = (i == p.first_key_chunk(m) ? SWEEP_INIT : 0) | (i == m ? SWEEP_FINAL : 0);
            { PROF(FPDT_PROF_FWD, st); launch_fwd_sweep(a, st); }
            ++t;
        }
        if (acth) {
            TRY(ev.record(EV_ACT_FREE0 + qbuf, st));
            TRY(ev.record(EV_OUT_DONE0 + qbuf, st));
            TRY(ev.wait(c->d2h, EV_OUT_DONE0 + qbuf));
            TRY(copy_d2h(O + (size_t)m * qb, f.o_buf[qbuf], qb, c->d2h));
            HIP_TRY(hipMemcpy2DAsync(LSE + m * p.C, (size_t)p.S * 4, f.lse_buf[qbuf], (size_t)p.C * 4,
                                     (size_t)p.C * 4, (size_t)p.Hq, hipMemcpyDeviceToHost, c->d2h));
            g_d2h_bytes += (size_t)p.C * 4 * p.Hq;
            TRY(ev.record(EV_OUT_COPIED0 + qbuf, c->d2h));
        }
    }
    if (c) {
        TRY(ev.record(EV_JOIN_H2D, c->h2d));
        TRY(ev.record(EV_JOIN_D2H, c->d2h));
        TRY(ev.wait(st, EV_JOIN_H2D));
        TRY(ev.wait(st, EV_JOIN_D2H));
    }
    return launch_status("bf16 pairwise forward");
}

// =========================================================================================
// backward
// =========================================================================================
int bwd_f32(const Problem& p, const float* Q, const float* K, const float* V, const float* O,
            const float* LSE, const float* dO, float* dQ, float* dK, float* dV, const BwdPlan& f,
            hipStream_t st)
{
    launch_zero(dQ, (size_t)p.S * p.Hq * p.D * 4, st);
    launch_zero(dK, (size_t)p.S * p.Hkv * p.D * 4, st);
    launch_zero(dV, (size_t)p.S * p.Hkv * p.D * 4, st);
    launch_delta(O, dO, p.S, p.Hq, p.D, 0, f.Delta, p.S, st);
    auto pair = [&](int64_t i, int64_t j) {
        F32BwdArgs a;
        a.Q = Q + (size_t)i * p.C * p.Hq * p.D;
        a.dO = dO + (size_t)i * p.C * p.Hq * p.D;
        a.K = K + (size_t)j * p.C * p.Hkv * p.D;
        a.V = V + (size_t)j * p.C * p.Hkv * p.D;
        a.LSE = LSE + i * p.C; a.Delta = f.Delta + i * p.C; a.row_stat_stride = p.S;
        a.dQ = dQ + (size_t)i * p.C * p.Hq * p.D;
        a.dK = dK + (size_t)j * p.C * p.Hkv * p.D;
        a.dV = dV + (size_t)j * p.C * p.Hkv * p.D;
        a.q_pos0 = i * p.C; a.k_pos0 = j * p.C; a.n_q = p.C; a.n_k = p.C;
        a.Hq = p.Hq; a.Hkv = p.Hkv; a.D = p.D; a.scale = p.scale;
        launch_f32_bwd_pair(a, st);
    };
    if (p.q_outer()) {
        for (int64_t i = 0; i < p.u; ++i)
            for (int64_t j = 0; j <= i; ++j)
                if (p.on(i, j)) pair(i, j);
    } else {
        for (int64_t j = 0; j < p.u; ++j)
            for (int64_t i = j; i < p.u; ++i)
                if (p.on(i, j)) pair(i, j);
    }
    return launch_status("fp32 backward");
}

int bwd_bf16_fused(const Problem& p, const void* Q, const void* K, const void* V, const void* O,
                   const float* LSE, const void* dO, void* dQ, void* dK, void* dV, const BwdPlan& f,
                   hipStream_t st)
{
    launch_delta(O, dO, p.S, p.Hq, p.D, 1, f.Delta, p.S, st);
    launch_delta_head(Q, dO, K, V, LSE, p.S, DELTA_HEAD_ROWS, p.Hq, p.Hkv, p.D, p.scale, f.Delta, st);
    launch_stat_pack(LSE, f.Delta, p.S, p.S, p.Hq, p.S / 32, f.stat2, st);
    launch_pack(Q, p.S, p.Hq, p.D, f.Qnat, nullptr, p.S / 32, st);
    launch_pack(dO, p.S, p.Hq, p.D, f.dOnat, nullptr, p.S / 32, st);
    launch_pack(K, p.S, p.Hkv, p.D, f.Knat, nullptr, p.S / 32, st);
    launch_pack(V, p.S, p.Hkv, p.D, f.Vnat, nullptr, p.S / 32, st);
    BwdArgs a;
    a.Q = Q; a.dO = dO; a.K = K; a.V = V;
    a.Qnat = f.Qnat; a.dOnat = f.dOnat; a.q_head_stride_blocks = p.S / 32;
    a.Knat = f.Knat; a.Vnat = f.Vnat; a.kv_head_stride_blocks = p.S / 32;
    a.LSE = LSE; a.Delta = f.Delta; a.row_stat_stride = p.S;
    a.stat2 = f.stat2;
    a.q_pos0 = 0; a.k_pos0 = 0; a.n_q = p.S; a.n_k = p.S;
    a.Hq = p.Hq; a.Hkv = p.Hkv; a.D = p.D; a.scale = p.scale;
    a.acc_dq = nullptr; a.acc_dk = nullptr; a.acc_dv = nullptr;
    a.dQ = dQ; a.dK = dK; a.dV = dV;
    a.flags = ACC_FINAL;
    { PROF(FPDT_PROF_DKDV, st); launch_bwd_dkdv(a, st); }
    { PROF(FPDT_PROF_DQ, st); launch_bwd_dq(a, st); }
    return launch_status("bf16 backward");
}

// Pair-by-pair backward in either loop order, with the streamed operands staged through
// double buffers.  Gradient accumulators stay in fp32 fragment order between pairs: the
// side held fixed by the outer loop needs one chunk of them, the other side one slot per
// chunk of the sequence.
int bwd_bf16_pairs(const Problem& p, const char* Q, const char* K, const char* V, const char* O,
                   const float* LSE, const char* dO, char* dQ, char* dK, char* dV, const BwdPlan& f,
                   hipStream_t st)
{
    const bool kvh = p.kv_host(), acth = p.act_host(), qo = p.q_outer();
    DeviceCtx* c = nullptr;
    CallEvents ev;
    if (kvh || acth) {
        TRY(get_ctx(&c));
        ev.c = c;
        TRY(ev.record(EV_FORK, st));
        TRY(ev.wait(c->h2d, EV_FORK));
        TRY(ev.wait(c->d2h, EV_FORK));
    }
    const size_t kvb = p.kv_chunk_bytes(), qb = p.q_chunk_bytes();
    const size_t acc_q_chunk = bwd_acc_dq_bytes(p.C, p.Hq, p.D) / 4;     // floats per chunk slot
    const size_t acc_kv_chunk = bwd_acc_dkv_bytes(p.C, p.Hkv, p.D) / 4;

    if (!acth) launch_delta(O, dO, p.S, p.Hq, p.D, 1, f.Delta, p.S, st);

    // pair order
    std::vector<std::pair<int64_t, int64_t>> pairs;  // (i = query chunk, j = key chunk)
    if (qo) {
        for (int64_t i = 0; i < p.u; ++i)
            for (int64_t j = 0; j <= i; ++j)
                if (p.on(i, j)) pairs.push_back({i, j});
    } else {
        for (int64_t j = 0; j < p.u; ++j)
            for (int64_t i = j; i < p.u; ++i)
                if (p.on(i, j)) pairs.push_back({i, j});
    }
    // K/V fetch sequence: one fetch whenever the key chunk changes
    std::vector<int64_t> kv_seq;
    for (size_t t = 0; t < pairs.size(); ++t)
        if (t == 0 || pairs[t].second != pairs[t - 1].second) kv_seq.push_back(pairs[t].second);

    auto fetch_kv = [&](size_t n) -> int {
        const int b = (int)(n & 1);
        TRY(ev.wait(c->h2d, EV_KV_FREE0 + b));
        TRY(copy_h2d(f.kv_raw[b], K + (size_t)kv_seq[n] * kvb, kvb, c->h2d));
        TRY(copy_h2d(f.kv_raw[b] + kvb, V + (size_t)kv_seq[n] * kvb, kvb, c->h2d));
        TRY(ev.record(EV_KV_READY0 + b, c->h2d));
        return FPDT_OK;
    };
    // activations (Q-outer only): Q_i, dO_i, O_i and the LSE strip of chunk i
    auto fetch_act = [&](int64_t i) -> int {
        const int b = (int)(i & 1);
        TRY(ev.wait(c->h2d, EV_ACT_FREE0 + b));
        TRY(copy_h2d(f.act_raw[b], Q + (size_t)i * qb, qb, c->h2d));
        TRY(copy_h2d(f.act_raw[b] + qb, dO + (size_t)i * qb, qb, c->h2d));
        TRY(copy_h2d(f.act_raw[b] + 2 * qb, O + (size_t)i * qb, qb, c->h2d));
        HIP_TRY(hipMemcpy2DAsync(f.lse_buf[b], (size_t)p.C * 4, LSE + i * p.C, (size_t)p.S * 4,
                                 (size_t)p.C * 4, (size_t)p.Hq, hipMemcpyHostToDevice, c->h2d));
        g_h2d_bytes += (size_t)p.C * 4 * p.Hq;
        TRY(ev.record(EV_ACT_READY0 + b, c->h2d));
        return FPDT_OK;
    };

    if (acth) TRY(fetch_act(0));
    if (kvh) TRY(fetch_kv(0));

    size_t kv_n = 0;         // index into kv_seq of the chunk currently staged
    int64_t cur_i = -1, cur_j = -1;
    const char *Qi = nullptr, *dOi = nullptr, *Kj = nullptr, *Vj = nullptr;
    const float *LSEi = nullptr, *Deltai = nullptr;
    int64_t stat_stride = p.S;
    bool stat_stale = true;  // f.stat2 does not hold the current query chunk's statistics yet
    for (size_t t = 0; t < pairs.size(); ++t) {
        const int64_t i = pairs[t].first, j = pairs[t].second;
        // both orders visit the key chunks of a query chunk, and the query chunks of a key chunk,
        // in ascending order: dQ_i starts at its first kept key chunk and ends on the diagonal,
        // dK_j / dV_j start on the diagonal and end at the last query chunk that keeps chunk j
        const bool last_for_q = (j == i);
        const bool last_for_kv = (i == p.last_query_chunk(j));
        const bool first_for_q = (j == p.first_key_chunk(i)), first_for_kv = (i == j);
        // ---- key/value side ----
        if (j != cur_j) {
            if (kvh) {
                if (cur_j >= 0) {  // previous staged chunk no longer read by any kernel
                    TRY(ev.record(EV_KV_FREE0 + (int)(kv_n & 1), st));
                    ++kv_n;
                }
                if (kv_n + 1 < kv_seq.size()) TRY(fetch_kv(kv_n + 1));
                const int b = (int)(kv_n & 1);
                TRY(ev.wait(st, EV_KV_READY0 + b));
                Kj = f.kv_raw[b];
                Vj = f.kv_raw[b] + kvb;
            } else {
                Kj = K + (size_t)j * kvb;
                Vj = V + (size_t)j * kvb;
            }
            launch_pack(Kj, p.C, p.Hkv, p.D, f.Knat, nullptr, p.C / 32, st);
            launch_pack(Vj, p.C, p.Hkv, p.D, f.Vnat, nullptr, p.C / 32, st);
            cur_j = j;
        }
        // ---- query side ----
        if (i != cur_i) {
            if (acth) {
                if (cur_i >= 0) TRY(ev.record(EV_ACT_FREE0 + (int)(cur_i & 1), st));
                if (i + 1 < p.u) TRY(fetch_act(i + 1));
                const int b = (int)(i & 1);
                TRY(ev.wait(st, EV_ACT_READY0 + b));
                Qi = f.act_raw[b];
                dOi = f.act_raw[b] + qb;
                launch_delta(f.act_raw[b] + 2 * qb, dOi, p.C, p.Hq, p.D, 1, f.delta_buf[b], p.C, st);
                LSEi = f.lse_buf[b];
                Deltai = f.delta_buf[b];
                stat_stride = p.C;
            } else {
                Qi = Q + (size_t)i * qb;
                dOi = dO + (size_t)i * qb;
                LSEi = LSE + i * p.C;
                Deltai = f.Delta + i * p.C;
                stat_stride = p.S;
            }
            launch_pack(Qi, p.C, p.Hq, p.D, f.Qnat, nullptr, p.C / 32, st);
            launch_pack(dOi, p.C, p.Hq, p.D, f.dOnat, nullptr, p.C / 32, st);
            cur_i = i;
            stat_stale = true;
        }
        // Rows that see only a few keys get their cancellation-safe Delta: the head of the
        // sequence (pair (0, 0)) and, with a chunk mask, the head of every query chunk that keeps
        // no earlier key chunk (its diagonal pair is then the first pair that reads its Delta).
        if (i == j && p.first_key_chunk(i) == i)
            launch_delta_head(Qi, dOi, Kj, Vj, LSEi, stat_stride, DELTA_HEAD_ROWS, p.Hq, p.Hkv, p.D,
                              p.scale, const_cast<float*>(Deltai), st);
        if (stat_stale) {  // after the head rows have their final Delta
            launch_stat_pack(LSEi, Deltai, stat_stride, p.C, p.Hq, p.C / 32, f.stat2, st);
            stat_stale = false;
        }
        // ---- the pair ----
        BwdArgs a;
        a.Q = Qi; a.dO = dOi; a.K = Kj; a.V = Vj;
        a.Qnat = f.Qnat; a.dOnat = f.dOnat; a.q_head_stride_blocks = p.C / 32;
        a.Knat = f.Knat; a.Vnat = f.Vnat; a.kv_head_stride_blocks = p.C / 32;
        a.LSE = LSEi; a.Delta = Deltai; a.row_stat_stride = stat_stride;
        a.stat2 = f.stat2;
        a.q_pos0 = i * p.C; a.k_pos0 = j * p.C; a.n_q = p.C; a.n_k = p.C;
        a.Hq = p.Hq; a.Hkv = p.Hkv; a.D = p.D; a.scale = p.scale;
        a.acc_dq = f.acc_dq + (qo ? 0 : (size_t)i * acc_q_chunk);
        a.acc_dk = f.acc_dk + (qo ? (size_t)j * acc_kv_chunk : 0);
        a.acc_dv = f.acc_dv + (qo ? (size_t)j * acc_kv_chunk : 0);
        const int ob_kv = (int)(j & 1), ob_q = (int)(i & 1);
        a.dK = kvh ? f.dkv_out[ob_kv] : dK + (size_t)j * kvb;
        a.dV = kvh ? f.dkv_out[ob_kv] + kvb : dV + (size_t)j * kvb;
        a.dQ = acth ? f.dq_out[ob_q] : dQ + (size_t)i * qb;
        a.dS_frag = f.ds_frag;  // null unless FPDT_BWD_STORE_DS: the dK/dV launch then writes the pair's dS tiles

        a.flags = (first_for_kv ? 0 : ACC_LOAD) | (last_for_kv ? ACC_FINAL : 0);
        if (kvh && last_for_kv) TRY(ev.wait(st, EV_DKV_COPIED0 + ob_kv));
        { PROF(FPDT_PROF_DKDV, st); launch_bwd_dkdv(a, st); }
        if (kvh && last_for_kv) {
            TRY(ev.record(EV_DKV_DONE0 + ob_kv, st));
            TRY(ev.wait(c->d2h, EV_DKV_DONE0 + ob_kv));
            TRY(copy_d2h(dK + (size_t)j * kvb, f.dkv_out[ob_kv], kvb, c->d2h));
            TRY(copy_d2h(dV + (size_t)j * kvb, f.dkv_out[ob_kv] + kvb, kvb, c->d2h));
            TRY(ev.record(EV_DKV_COPIED0 + ob_kv, c->d2h));
        }

        a.flags = (first_for_q ? 0 : ACC_LOAD) | (last_for_q ? ACC_FINAL : 0);
        if (acth && last_for_q) TRY(ev.wait(st, EV_OUT_COPIED0 + ob_q));
        {
            PROF(FPDT_PROF_DQ, st);
            if (a.dS_frag) launch_bwd_dq_from_ds(a, st);  // one GEMM on the tiles just written
            else launch_bwd_dq(a, st);
        }
        if (acth && last_for_q) {
            TRY(ev.record(EV_OUT_DONE0 + ob_q, st));
            TRY(ev.wait(c->d2h, EV_OUT_DONE0 + ob_q));
            TRY(copy_d2h(dQ + (size_t)i * qb, f.dq_out[ob_q], qb, c->d2h));
            TRY(ev.record(EV_OUT_COPIED0 + ob_q, c->d2h));
        }
    }
    if (c) {
        TRY(ev.record(EV_JOIN_H2D, c->h2d));
        TRY(ev.record(EV_JOIN_D2H, c->d2h));
        TRY(ev.wait(st, EV_JOIN_H2D));
        TRY(ev.wait(st, EV_JOIN_D2H));
    }
    return launch_status("bf16 pairwise backward");
}

}  // namespace

// =========================================================================================
// exported entry points
// =========================================================================================
extern "C" {

size_t fpdt_attn_workspace_bytes(int64_t S, int64_t chunk, int Hq, int Hkv, int D, int dtype,
                                 unsigned flags, int is_bwd)
{
    Problem p;
    if (!is_bwd) flags &= ~(unsigned)FPDT_BWD_STORE_DS;  // backward-only flag
    if (validate_scalars(p, S, chunk, Hq, Hkv, D, 1.f, dtype, flags) != FPDT_OK) return 0;
    return is_bwd ? plan_bwd(p, nullptr).total : plan_fwd(p, nullptr).total;
}

int64_t fpdt_attn_pick_chunk(int64_t S, int Hq, int Hkv, int D, int dtype, unsigned flags,
                             size_t max_workspace_bytes)
{
    g_err.clear();
    const int64_t step = dtype == FPDT_DTYPE_BF16 ? FPDT_CHUNK_MULTIPLE : 1;
    // The measured throughput curve is flat from 32K tokens on and gains 0.3% at most beyond 64K,
    // while every chunk buffer, packed operand buffer and carried-state slot doubles with the
    // chunk: the knee, not the largest chunk that fits, is the target.
    const int64_t cap = FPDT_PREFERRED_CHUNK;
    auto fits = [&](int64_t c) {
        Problem q;
        if (validate_scalars(q, S, c, Hq, Hkv, D, 1.f, dtype, flags) != FPDT_OK) return false;
        if (!max_workspace_bytes) return true;
        return plan_fwd(q, nullptr).total <= max_workspace_bytes && plan_bwd(q, nullptr).total <= max_workspace_bytes;
    };
    // divisors of S that are multiples of `step`, from the cap downwards: the first that fits
    for (int64_t c = (S < cap ? S : cap) / step * step; c >= step; c -= step) {
        if (S % c == 0 && fits(c)) { g_err.clear(); return c; }
    }
    Problem q;  // say why: the arguments themselves, or the workspace limit
    if (validate_scalars(q, S, step, Hq, Hkv, D, 1.f, dtype, flags) == FPDT_OK || S % step != 0) {
        if (S > 0 && S % step != 0) fail(FPDT_ERR_UNSUPPORTED, "S=%lld has no chunk size that is a multiple of %lld", (long long)S, (long long)step);
        else fail(FPDT_ERR_WORKSPACE, "no chunk size of S=%lld fits in %zu bytes of workspace", (long long)S, max_workspace_bytes);
    }
    return 0;
}

static int attn_fwd_impl(const void* Q, const void* K, const void* V, void* O, float* LSE, int64_t S,
                         int64_t chunk, int Hq, int Hkv, int D, float scale, int dtype, unsigned flags,
                         const unsigned char* chunk_mask, bool sparse, void* workspace,
                         size_t workspace_bytes, void* stream, bool static_workspace = false)
{
    g_err.clear();
    g_h2d_bytes = g_d2h_bytes = 0;
    if (!Q || !K || !V || !O || !LSE) return fail(FPDT_ERR_INVALID_ARG, "NULL tensor pointer");
    flags &= ~(unsigned)FPDT_BWD_STORE_DS;  // backward-only flag
    Problem p;
    TRY(validate_scalars(p, S, chunk, Hq, Hkv, D, scale, dtype, flags));
    if (sparse) TRY(take_mask(p, chunk_mask));
    const size_t need = plan_fwd(p, nullptr).total;
    if (static_workspace) {
        if (need > workspace_bytes)
            return fail(FPDT_ERR_WORKSPACE, "these sizes need %zu bytes of workspace; the built-in scratch array of fpdt_attn_fwd_noalloc holds %zu (use fpdt_attn_fwd with a workspace of your own)", need, workspace_bytes);
    } else if (need && (!workspace || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 256))
        TRY(check_workspace(workspace, workspace_bytes, need));
    const size_t qbytes = (size_t)S * Hq * D * p.esize(), kbytes = (size_t)S * Hkv * D * p.esize();
    TRY(check_ptr(Q, qbytes, p.act_host(), "Q"));
    TRY(check_ptr(K, kbytes, p.kv_host(), "K"));
    TRY(check_ptr(V, kbytes, p.kv_host(), "V"));
    TRY(check_ptr(O, qbytes, p.act_host(), "O"));
    TRY(check_ptr(LSE, (size_t)S * Hq * 4, p.act_host(), "LSE"));
    // (the static array is not in HIP's allocation table: its size and alignment are known)
    if (!static_workspace) TRY(check_workspace(workspace, workspace_bytes, need));
    const FwdPlan f = plan_fwd(p, workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g_mu);
    if (!p.bf16())
        return fwd_f32(p, (const float*)Q, (const float*)K, (const float*)V, (float*)O, LSE, f, st);
    if (p.fused()) return fwd_bf16_fused(p, Q, K, V, O, LSE, f, st);
    return fwd_bf16_pairs(p, (const char*)Q, (const char*)K, (const char*)V, (char*)O, LSE, f, st);
}

int fpdt_attn_fwd(const void* Q, const void* K, const void* V, void* O, float* LSE, int64_t S,
                  int64_t chunk, int Hq, int Hkv, int D, float scale, int dtype, unsigned flags,
                  void* workspace, size_t workspace_bytes, void* stream)
{
    return attn_fwd_impl(Q, K, V, O, LSE, S, chunk, Hq, Hkv, D, scale, dtype, flags, nullptr, false,
                         workspace, workspace_bytes, stream);
}

int fpdt_attn_fwd_noalloc(const void* Q, const void* K, const void* V, void* O, float* LSE, int64_t S,
                          int64_t chunk, int Hq, int Hkv, int D, float scale, int dtype, unsigned flags,
                          void* stream)
{
    g_err.clear();
    // the offload schedules create their side streams and events on first use
    if (flags & (FPDT_KV_ON_HOST | FPDT_ACT_ON_HOST))
        return fail(FPDT_ERR_UNSUPPORTED, "fpdt_attn_fwd_noalloc takes resident tensors only (no offload flags)");
    void* ws = nullptr;
    TRY(scratch_for_current_device(&ws));
    g_no_alloc_call = true;
    const int rc = attn_fwd_impl(Q, K, V, O, LSE, S, chunk, Hq, Hkv, D, scale, dtype, flags, nullptr, false,
                                 ws, (size_t)FPDT_NOALLOC_SCRATCH_BYTES, stream, true);
    g_no_alloc_call = false;
    return rc;
}

int fpdt_attn_fwd_blocksparse(const void* Q, const void* K, const void* V, void* O, float* LSE,
                              int64_t S, int64_t chunk, int Hq, int Hkv, int D, float scale, int dtype,
                              unsigned flags, const unsigned char* chunk_mask, void* workspace,
                              size_t workspace_bytes, void* stream)
{
    return attn_fwd_impl(Q, K, V, O, LSE, S, chunk, Hq, Hkv, D, scale, dtype, flags | FPDT_PAIRWISE,
                         chunk_mask, true, workspace, workspace_bytes, stream);
}

static int attn_bwd_impl(const void* Q, const void* K, const void* V, const void* O, const float* LSE,
                         const void* dO, void* dQ, void* dK, void* dV, int64_t S, int64_t chunk, int Hq,
                         int Hkv, int D, float scale, int dtype, unsigned flags,
                         const unsigned char* chunk_mask, bool sparse, void* workspace,
                         size_t workspace_bytes, void* stream)
{
    g_err.clear();
    g_h2d_bytes = g_d2h_bytes = 0;
    if (!Q || !K || !V || !O || !LSE || !dO || !dQ || !dK || !dV)
        return fail(FPDT_ERR_INVALID_ARG, "NULL tensor pointer");
    Problem p;
    TRY(validate_scalars(p, S, chunk, Hq, Hkv, D, scale, dtype, flags));
    if (sparse) TRY(take_mask(p, chunk_mask));
    const size_t need = plan_bwd(p, nullptr).total;
    if (need && (!workspace || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 256))
        TRY(check_workspace(workspace, workspace_bytes, need));
    const size_t qbytes = (size_t)S * Hq * D * p.esize(), kbytes = (size_t)S * Hkv * D * p.esize();
    TRY(check_ptr(Q, qbytes, p.act_host(), "Q"));
    TRY(check_ptr(O, qbytes, p.act_host(), "O"));
    TRY(check_ptr(dO, qbytes, p.act_host(), "dO"));
    TRY(check_ptr(dQ, qbytes, p.act_host(), "dQ"));
    TRY(check_ptr(LSE, (size_t)S * Hq * 4, p.act_host(), "LSE"));
    TRY(check_ptr(K, kbytes, p.kv_host(), "K"));
    TRY(check_ptr(V, kbytes, p.kv_host(), "V"));
    TRY(check_ptr(dK, kbytes, p.kv_host(), "dK"));
    TRY(check_ptr(dV, kbytes, p.kv_host(), "dV"));
    TRY(check_workspace(workspace, workspace_bytes, need));
    const BwdPlan f = plan_bwd(p, workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    std::lock_guard<std::mutex> lock(g_mu);
    if (!p.bf16())
        return bwd_f32(p, (const float*)Q, (const float*)K, (const float*)V, (const float*)O, LSE,
                       (const float*)dO, (float*)dQ, (float*)dK, (float*)dV, f, st);
    if (p.fused()) return bwd_bf16_fused(p, Q, K, V, O, LSE, dO, dQ, dK, dV, f, st);
    return bwd_bf16_pairs(p, (const char*)Q, (const char*)K, (const char*)V, (const char*)O, LSE,
                          (const char*)dO, (char*)dQ, (char*)dK, (char*)dV, f, st);
}

int fpdt_attn_bwd(const void* Q, const void* K, const void* V, const void* O, const float* LSE,
                  const void* dO, void* dQ, void* dK, void* dV, int64_t S, int64_t chunk, int Hq,
                  int Hkv, int D, float scale, int dtype, unsigned flags, void* workspace,
                  size_t workspace_bytes, void* stream)
{
    return attn_bwd_impl(Q, K, V, O, LSE, dO, dQ, dK, dV, S, chunk, Hq, Hkv, D, scale, dtype, flags,
                         nullptr, false, workspace, workspace_bytes, stream);
}

int fpdt_attn_bwd_blocksparse(const void* Q, const void* K, const void* V, const void* O,
                              const float* LSE, const void* dO, void* dQ, void* dK, void* dV, int64_t S,
                              int64_t chunk, int Hq, int Hkv, int D, float scale, int dtype,
                              unsigned flags, const unsigned char* chunk_mask, void* workspace,
                              size_t workspace_bytes, void* stream)
{
    return attn_bwd_impl(Q, K, V, O, LSE, dO, dQ, dK, dV, S, chunk, Hq, Hkv, D, scale, dtype,
                         flags | FPDT_PAIRWISE, chunk_mask, true, workspace, workspace_bytes, stream);
}

int fpdt_attn_merge(const void* O_a, const float* LSE_a, const void* O_b, const float* LSE_b,
                    void* O_out, float* LSE_out, int64_t rows, int Hq, int D, int dtype, void* stream)
{
    g_err.clear();
    if (!O_a || !LSE_a || !O_b || !LSE_b || !O_out || !LSE_out) return fail(FPDT_ERR_INVALID_ARG, "NULL pointer");
    if (rows <= 0 || Hq <= 0 || D <= 0) return fail(FPDT_ERR_INVALID_ARG, "rows, Hq and D must be positive");
    if (dtype != FPDT_DTYPE_F32 && dtype != FPDT_DTYPE_BF16) return fail(FPDT_ERR_INVALID_ARG, "unknown dtype %d", dtype);
    if (rows * Hq > ((int64_t)1 << 34)) return fail(FPDT_ERR_UNSUPPORTED, "too many rows");
    const size_t ob = (size_t)rows * Hq * D * (dtype == FPDT_DTYPE_BF16 ? 2 : 4), lb = (size_t)rows * Hq * 4;
    TRY(check_ptr(O_a, ob, false, "O_a"));
    TRY(check_ptr(O_b, ob, false, "O_b"));
    TRY(check_ptr(O_out, ob, false, "O_out"));
    TRY(check_ptr(LSE_a, lb, false, "LSE_a"));
    TRY(check_ptr(LSE_b, lb, false, "LSE_b"));
    TRY(check_ptr(LSE_out, lb, false, "LSE_out"));
    launch_merge(O_a, LSE_a, O_b, LSE_b, O_out, LSE_out, rows, Hq, D, dtype == FPDT_DTYPE_BF16,
                 static_cast<hipStream_t>(stream));
    return launch_status("merge");
}

int fpdt_last_link_bytes(uint64_t* h2d_bytes, uint64_t* d2h_bytes)
{
    if (h2d_bytes) *h2d_bytes = g_h2d_bytes;
    if (d2h_bytes) *d2h_bytes = g_d2h_bytes;
    return FPDT_OK;
}

int fpdt_profile_enable(int on)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof_on = on != 0;
    return FPDT_OK;
}

int fpdt_profile_read(int kind, double* total_ms, int64_t* launches)
{
    if (kind < 0 || kind >= FPDT_PROF_KINDS) return fail(FPDT_ERR_INVALID_ARG, "unknown profile kind %d", kind);
    std::lock_guard<std::mutex> lk(g_prof_mu);
    double ms = 0.0;
    int64_t n = 0;
    std::vector<ProfRec> keep;
    for (const ProfRec& r : g_prof) {
        if (r.kind != kind) { keep.push_back(r); continue; }
        float t = 0.f;
        hipError_t e = hipEventSynchronize(r.b);
        if (e == hipSuccess) e = hipEventElapsedTime(&t, r.a, r.b);
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
        if (e != hipSuccess) { g_prof.swap(keep); return fail(FPDT_ERR_HIP, "profile events: %s", hipGetErrorString(e)); }
        ms += t;
        ++n;
    }
    g_prof.swap(keep);
    if (total_ms) *total_ms = ms;
    if (launches) *launches = n;
    return FPDT_OK;
}

int fpdt_calibrate_mfma(int kind, int iters, void* workspace, size_t workspace_bytes, double* tflops,
                        double* ms, void* stream)
{
    g_err.clear();
    if (kind < 0 || kind >= FPDT_CAL_KINDS) return fail(FPDT_ERR_INVALID_ARG, "unknown calibration kind %d", kind);
    if (iters < 1 || iters > 1000000) return fail(FPDT_ERR_INVALID_ARG, "iters must be in 1 .. 1000000");
    if (!tflops) return fail(FPDT_ERR_INVALID_ARG, "tflops is NULL");
    TRY(check_workspace(workspace, workspace_bytes, FPDT_CAL_WORKSPACE_BYTES));
    int dev = 0, cus = 0;
    HIP_TRY(hipGetDevice(&dev));
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    if (cus < 1 || (size_t)cus * 512 * 4 + 4096 > FPDT_CAL_WORKSPACE_BYTES) return fail(FPDT_ERR_UNSUPPORTED, "%d compute units", cus);
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* base = static_cast<char*>(workspace);
    float* out = reinterpret_cast<float*>(base + 4096);
    launch_calibrate_fill(base, st);
    const int warm = iters / 50 > 0 ? iters / 50 : 1;
    const int waves = launch_calibrate(kind, out, base, warm, cus, st);
    TRY(launch_status("calibration warm-up"));
    hipEvent_t a = nullptr, b = nullptr;
    HIP_TRY(hipEventCreate(&a));
    hipError_t e = hipEventCreate(&b);
    if (e == hipSuccess) e = hipEventRecord(a, st);
    if (e == hipSuccess) {
        launch_calibrate(kind, out, base, iters, cus, st);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipEventRecord(b, st);
    if (e == hipSuccess) e = hipEventSynchronize(b);
    float t = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&t, a, b);
    (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
    if (e != hipSuccess) return fail(FPDT_ERR_HIP, "calibration run: %s", hipGetErrorString(e));
    const double flops = (double)cus * 4.0 * waves * (double)iters * CALIBRATE_MFMA_PER_TRIP * (2.0 * 32 * 32 * 16);
    *tflops = flops / (t * 1e-3) / 1e12;
    if (ms) *ms = t;
    return FPDT_OK;
}

int fpdt_debug_configure(unsigned flags)
{
    g_err.clear();
    if (flags & ~(unsigned)(FPDT_DEBUG_POISON_STAGING | FPDT_DEBUG_DELAY_COPIES))
        return fail(FPDT_ERR_INVALID_ARG, "unknown debug flag bits 0x%x", flags);
    std::lock_guard<std::mutex> lock(g_mu);
    if (flags & FPDT_DEBUG_DELAY_COPIES) {
        DeviceCtx* c = nullptr;
        TRY(get_ctx(&c));
        if (!c->delay_host) {
            void* h = nullptr;
            HIP_TRY(hipHostMalloc(&h, DELAY_BYTES, hipHostMallocDefault));
            memset(h, 0, DELAY_BYTES);
            if (!c->delay_dev) {
                hipError_t e = hipMalloc(&c->delay_dev, DELAY_BYTES);
                if (e != hipSuccess) {
                    (void)hipHostFree(h);
                    return fail(FPDT_ERR_HIP, "hipMalloc of the delay buffer failed: %s", hipGetErrorString(e));
                }
            }
            c->delay_host = h;
        }
    }
    g_debug = flags;
    return FPDT_OK;
}

const char* fpdt_last_error(void) { return g_err.c_str(); }

const char* fpdt_version(void) { return "fpdt 0.1 gfx950"; }

}  // extern "C"
