// C ABI of libmoe_hip.so: argument validation on the host, then kernel launches
// on the caller's stream.  See include/moe.h for the contract of each call.
#include "moe_internal.h"
#include "moe_measure.h"

// Scratch of moe_layer_static: what the other entry points take as `workspace`, in a static device
// array.  Every device the library runs on holds its own copy at its own address; in host code the
// name below is only a handle for hipGetSymbolAddress, which static_scratch() calls once per device
// and whose result is what kernels, copies and carve() get.  (No __attribute__((used)) here: with it
// the compiler keeps the device-side variable at internal linkage, the code object then exports no
// such symbol and the runtime aborts in the lookup.  The reference from host code below is what makes
// the compiler export it.)
static __device__ __align__(256) unsigned char scratch[MOE_STATIC_SCRATCH_BYTES];

namespace moe {

static size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

WorkspaceLayout workspace_layout(const moe_shape_t& s, int tokens) {
    WorkspaceLayout L{};
    const size_t nb = (size_t)route_blocks(tokens > 0 ? tokens : 1);
    const size_t A = (size_t)(tokens > 0 ? tokens : 1) * (size_t)s.top_k;
    const size_t esz = s.dtype == MOE_F32 ? 4 : 2;
    size_t off = 0;
    L.dec_flags = off;   off = align_up(off + kDecodeFlagInts * sizeof(uint32_t));
    L.sync = off;        off = align_up(off + kSyncInts * sizeof(int32_t));
    L.hist = off;        off = align_up(off + nb * s.n_experts * sizeof(int32_t));
    L.hist_next = off;   off = align_up(off + nb * s.n_experts * sizeof(int32_t));
    L.offs = off;        off = align_up(off + (size_t)(s.n_experts + 1) * sizeof(int32_t));
    L.row_of_slot = off; off = align_up(off + A * sizeof(int32_t));
    L.slot_of = off;     off = align_up(off + A * sizeof(int32_t));
    L.route_end = off;
    L.act = off;         off = align_up(off + A * (size_t)s.ffn * esz);
    L.out = off;         off = align_up(off + A * (size_t)s.hidden * sizeof(float));
    L.partial = off;
    if (s.dtype == MOE_BF16 && tokens > kStreamMaxTokens) off = align_up(off + kGemmScratchBytes);
    L.total = off;
    return L;
}

// ---- optional per-stage timing ------------------------------------------------
namespace {
struct StageTimer {
    static constexpr int kMaxMarks = 8;
    int max_calls = 0, calls = 0;
    int cur = -1;  // index of the call being recorded
    hipEvent_t* events = nullptr;  // [max_calls][kMaxMarks]
    int* stage_of = nullptr;       // [max_calls][kMaxMarks], -1 = call start
    int* n_marks = nullptr;        // [max_calls]
};
thread_local StageTimer* g_timer = nullptr;

void stage_call_begin(hipStream_t stream) {
    StageTimer* t = g_timer;
    if (t == nullptr) return;
    if (t->calls >= t->max_calls) {
        t->cur = -1;
        return;
    }
    t->cur = t->calls++;
    t->n_marks[t->cur] = 1;
    t->stage_of[t->cur * StageTimer::kMaxMarks] = -1;
    (void)hipEventRecord(t->events[t->cur * StageTimer::kMaxMarks], stream);
}
}  // namespace

void stage_mark(hipStream_t stream, int stage) {
    StageTimer* t = g_timer;
    if (t == nullptr || t->cur < 0) return;
    int& n = t->n_marks[t->cur];
    if (n >= StageTimer::kMaxMarks) return;
    t->stage_of[t->cur * StageTimer::kMaxMarks + n] = stage;
    (void)hipEventRecord(t->events[t->cur * StageTimer::kMaxMarks + n], stream);
    ++n;
}

namespace {
int g_decode_spin_limit = 1 << 22;

constexpr int kMaxDevices = 64;
void* g_static_scratch[kMaxDevices] = {nullptr};

// Device address of `scratch` on the current device, looked up once per device.
void* static_scratch() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    if (g_static_scratch[dev] == nullptr) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_static_scratch[dev] = ptr;   // a race between threads stores the same address twice
    }
    return g_static_scratch[dev];
}
}
int decode_spin_limit() { return g_decode_spin_limit; }

int compute_units() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

namespace {

constexpr int kMaxTokens = 1 << 20;

int check_shape(const moe_shape_t* s) {
    if (s == nullptr) return MOE_ERR_NULL;
    if (s->dtype != MOE_F32 && s->dtype != MOE_BF16) return MOE_ERR_DTYPE;
    if (s->reserved != 0) return MOE_ERR_SHAPE;
    if (s->hidden <= 0 || s->ffn <= 0 || s->hidden % 64 != 0 || s->ffn % 64 != 0) return MOE_ERR_SHAPE;
    if (s->n_experts < 1 || s->n_experts > 64) return MOE_ERR_SHAPE;
    if (s->top_k < 1 || s->top_k > 8 || s->top_k > s->n_experts) return MOE_ERR_SHAPE;
    return MOE_OK;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Returns MOE_ERR_NULL / MOE_ERR_ALIGN for a list of required pointers.
template <size_t N>
int check_required(const void* const (&ptrs)[N]) {
    for (const void* p : ptrs)
        if (p == nullptr) return MOE_ERR_NULL;
    for (const void* p : ptrs)
        if (misaligned(p)) return MOE_ERR_ALIGN;
    return MOE_OK;
}

template <size_t N>
int check_optional(const void* const (&ptrs)[N]) {
    for (const void* p : ptrs)
        if (p != nullptr && misaligned(p)) return MOE_ERR_ALIGN;
    return MOE_OK;
}

int dev(hipError_t e) { return e == hipSuccess ? MOE_OK : MOE_ERR_DEVICE; }

// bf16 calls of at most kDecodeMaxTokens tokens run as one kernel (routing included); up to
// kStreamMaxTokens the expert FFN still uses that kernel's weight-streaming phases.
bool decode_path(const moe_shape_t& s, int tokens) { return s.dtype == MOE_BF16 && tokens <= kDecodeMaxTokens; }
bool stream_path(const moe_shape_t& s, int tokens) { return s.dtype == MOE_BF16 && tokens <= kStreamMaxTokens; }

struct Ws {
    int32_t *hist, *hist_next, *offs, *row_of_slot, *slot_of, *sync;
    uint32_t* dec_flags;
    void* act;
    float* out;
    float* partial;
};

Ws carve(void* workspace, const WorkspaceLayout& L) {
    char* b = static_cast<char*>(workspace);
    Ws w;
    w.hist = reinterpret_cast<int32_t*>(b + L.hist);
    w.hist_next = reinterpret_cast<int32_t*>(b + L.hist_next);
    w.offs = reinterpret_cast<int32_t*>(b + L.offs);
    w.row_of_slot = reinterpret_cast<int32_t*>(b + L.row_of_slot);
    w.slot_of = reinterpret_cast<int32_t*>(b + L.slot_of);
    w.sync = reinterpret_cast<int32_t*>(b + L.sync);
    w.dec_flags = reinterpret_cast<uint32_t*>(b + L.dec_flags);
    w.act = b + L.act;
    w.out = reinterpret_cast<float*>(b + L.out);
    w.partial = reinterpret_cast<float*>(b + L.partial);
    return w;
}

// Routing for one or two gates.  With `permute`, also leaves offs / row_of_slot / slot_of in
// the workspace for the grouped GEMMs.
hipError_t run_route(const moe_shape_t& s, int tokens, const void* x, GateArgs* gates, int n_gates, int32_t* counts,
                     int accumulate, int32_t* counts_next, bool permute, const Ws& ws, hipStream_t stream) {
    if (tokens <= kDecodeMaxTokens) {
        // Decode-size calls: one workgroup routes every token and writes the counts itself.
        hipError_t e = launch_route_small(s, tokens, x, gates, n_gates, counts, accumulate, counts_next, stream);
        stage_mark(stream, kStageRoute);
        if (e != hipSuccess || !permute) return e;
        e = launch_hist_from_idx(s, tokens, gates[0].idx, ws.hist, stream);
        if (e != hipSuccess) return e;
        e = launch_finalize(s, tokens, ws.hist, gates[0].idx, nullptr, 0, ws.offs, ws.row_of_slot, ws.slot_of, ws.sync, stream);
        stage_mark(stream, kStagePermute);
        return e;
    }
    gates[0].hist = ws.hist;
    if (n_gates > 1) gates[1].hist = counts_next != nullptr ? ws.hist_next : nullptr;
    hipError_t e = launch_route(s, tokens, x, gates, n_gates, stream);
    stage_mark(stream, kStageRoute);
    if (e != hipSuccess) return e;
    if (counts != nullptr || permute)  // (a caller whose expert kernel counts the selections itself passes neither)
        e = launch_finalize(s, tokens, ws.hist, gates[0].idx, counts, accumulate, permute ? ws.offs : nullptr,
                            permute ? ws.row_of_slot : nullptr, permute ? ws.slot_of : nullptr,
                            permute ? ws.sync : nullptr, stream);
    if (e != hipSuccess) return e;
    if (n_gates > 1 && counts_next != nullptr)
        e = launch_finalize(s, tokens, ws.hist_next, gates[1].idx, counts_next, 0, nullptr, nullptr, nullptr, nullptr, stream);
    stage_mark(stream, kStagePermute);
    return e;
}

constexpr StaleInput kNoStaleInput = {nullptr, nullptr};

hipError_t run_ffn(const moe_shape_t& s, int tokens, const void* x, const int32_t* idx, const float* w,
                   const void* w1, const void* w3, const void* w2, void* y, const Ws& ws, hipStream_t stream,
                   const StaleInput& alt = kNoStaleInput, int32_t* counts = nullptr, int accumulate = 0) {
    if (stream_path(s, tokens))
        return launch_decode_layer(s, tokens, x, nullptr, idx, w, w1, w3, w2, y, ws.act, ws.dec_flags, alt, stream, counts,
                                   accumulate);
    if (s.dtype == MOE_F32)
        return launch_ffn_f32(s, tokens, static_cast<const float*>(x), w, static_cast<const float*>(w1),
                              static_cast<const float*>(w3), static_cast<const float*>(w2), static_cast<float*>(y),
                              ws.offs, ws.row_of_slot, ws.slot_of, static_cast<float*>(ws.act), ws.out, alt, stream);
    return launch_ffn_bf16(s, tokens, x, w, w1, w3, w2, y, ws.offs, ws.row_of_slot, ws.slot_of, ws.act, ws.out,
                           ws.sync, ws.partial, alt, stream);
}

// Expert execution on a carved workspace from selections made earlier (arguments already checked).
int enqueue_expert_ffn(const moe_shape_t& s, int32_t tokens, const void* x, const int32_t* topk_idx, const float* topk_w,
                       const void* w1, const void* w3, const void* w2, void* y, const Ws& ws, hipStream_t stream,
                       const StaleInput& alt) {
    stage_call_begin(stream);
    if (!stream_path(s, tokens)) {
        hipError_t e = launch_hist_from_idx(s, tokens, topk_idx, ws.hist, stream);
        if (e != hipSuccess) return MOE_ERR_DEVICE;
        e = launch_finalize(s, tokens, ws.hist, topk_idx, nullptr, 0, ws.offs, ws.row_of_slot, ws.slot_of, ws.sync, stream);
        stage_mark(stream, kStagePermute);
        if (e != hipSuccess) return MOE_ERR_DEVICE;
    }
    return dev(run_ffn(s, tokens, x, topk_idx, topk_w, w1, w3, w2, y, ws, stream, alt));
}


// Argument checks of a whole-layer call, everything but the workspace.
int check_layer_args(const moe_shape_t* shape, int32_t tokens, const void* x, const void* w_gate, const float* gate_bias,
                     const void* w_gate_next, const float* gate_bias_next, const void* w1, const void* w3, const void* w2,
                     void* y, int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* pred_idx) {
    if (int rc = check_shape(shape)) return rc;
    if (tokens < 0 || tokens > kMaxTokens) return MOE_ERR_SHAPE;
    const void* const req[] = {w_gate, w1, w3, w2, counts};
    if (int rc = check_required(req)) return rc;
    const void* const per_token[] = {x, y, topk_idx, topk_w};
    if (int rc = tokens > 0 ? check_required(per_token) : check_optional(per_token)) return rc;
    if (tokens > 0 && w_gate_next != nullptr && pred_idx == nullptr) return MOE_ERR_NULL;
    const void* const opt[] = {gate_bias, w_gate_next, gate_bias_next, pred_idx};
    return check_optional(opt);
}

// The kernels of one whole layer on a carved workspace (arguments already checked).
int enqueue_layer(const moe_shape_t& s, int32_t tokens, const void* x, const void* w_gate, const float* gate_bias,
                  const void* w_gate_next, const float* gate_bias_next, const void* w1, const void* w3, const void* w2,
                  void* y, int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t accumulate, int32_t* pred_idx,
                  const Ws& ws, hipStream_t stream) {
    if (tokens == 0)
        return dev(launch_finalize(s, 0, ws.hist, nullptr, counts, accumulate, nullptr, nullptr, nullptr, nullptr, stream));
    stage_call_begin(stream);
    if (decode_path(s, tokens)) {
        // One kernel routes, runs the experts and (in one of its workgroups, at the end) evaluates the
        // prediction gate.
        const DecodeRoute r = {w_gate, gate_bias, topk_idx, topk_w, counts, accumulate, w_gate_next, gate_bias_next, pred_idx};
        return dev(launch_decode_layer(s, tokens, x, &r, nullptr, nullptr, w1, w3, w2, y, ws.act, ws.dec_flags, kNoStaleInput,
                                       stream));
    }
    GateArgs g[2] = {{w_gate, gate_bias, topk_idx, topk_w, nullptr}, {w_gate_next, gate_bias_next, pred_idx, nullptr, nullptr}};
    const int n_gates = w_gate_next != nullptr ? 2 : 1;
    // 17 to 32 tokens: the weight-streaming kernel needs no permutation and counts the selections itself.
    const bool streaming = stream_path(s, tokens);
    hipError_t e = run_route(s, tokens, x, g, n_gates, streaming ? nullptr : counts, accumulate, nullptr, !streaming, ws, stream);
    if (e != hipSuccess) return MOE_ERR_DEVICE;
    return dev(run_ffn(s, tokens, x, topk_idx, topk_w, w1, w3, w2, y, ws, stream, kNoStaleInput, streaming ? counts : nullptr,
                       accumulate));
}

}  // namespace
}  // namespace moe

using namespace moe;

extern "C" {

const char* moe_status_string(int status) {
    switch (status) {
        case MOE_OK: return "ok";
        case MOE_ERR_NULL: return "a required pointer is NULL";
        case MOE_ERR_SHAPE: return "a dimension is outside the supported limits";
        case MOE_ERR_DTYPE: return "unsupported dtype";
        case MOE_ERR_WORKSPACE: return "workspace too small";
        case MOE_ERR_ALIGN: return "a pointer is not 16-byte aligned";
        case MOE_ERR_DEVICE: return "kernel launch failed";
        case MOE_ERR_TOO_LARGE: return "the call needs more scratch than the library's static buffer holds";
        default: return "unknown status";
    }
}

int moe_workspace_bytes(const moe_shape_t* shape, int32_t max_tokens, size_t* out_bytes) {
    if (out_bytes == nullptr) return MOE_ERR_NULL;
    if (int rc = check_shape(shape)) return rc;
    if (max_tokens < 0 || max_tokens > kMaxTokens) return MOE_ERR_SHAPE;
    *out_bytes = workspace_layout(*shape, max_tokens).total;
    return MOE_OK;
}

int moe_route_workspace_bytes(const moe_shape_t* shape, int32_t max_tokens, size_t* out_bytes) {
    if (out_bytes == nullptr) return MOE_ERR_NULL;
    if (int rc = check_shape(shape)) return rc;
    if (max_tokens < 0 || max_tokens > kMaxTokens) return MOE_ERR_SHAPE;
    *out_bytes = workspace_layout(*shape, max_tokens).route_end;
    return MOE_OK;
}

int moe_route(const moe_shape_t* shape, int32_t tokens, const void* x, const void* w_gate, const float* gate_bias,
              int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t accumulate, void* workspace,
              size_t workspace_bytes, void* hip_stream) {
    if (int rc = check_shape(shape)) return rc;
    if (tokens < 0 || tokens > kMaxTokens) return MOE_ERR_SHAPE;
    const void* const req[] = {w_gate, counts, workspace};
    if (int rc = check_required(req)) return rc;
    const void* const per_token[] = {x, topk_idx, topk_w};
    if (int rc = tokens > 0 ? check_required(per_token) : check_optional(per_token)) return rc;
    const void* const opt[] = {gate_bias};
    if (int rc = check_optional(opt)) return rc;
    const WorkspaceLayout L = workspace_layout(*shape, tokens);
    if (workspace_bytes < L.route_end) return MOE_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const Ws ws = carve(workspace, L);
    if (tokens == 0)
        return dev(launch_finalize(*shape, 0, ws.hist, nullptr, counts, accumulate, nullptr, nullptr, nullptr, nullptr, stream));
    stage_call_begin(stream);
    GateArgs g[1] = {{w_gate, gate_bias, topk_idx, topk_w, nullptr}};
    return dev(run_route(*shape, tokens, x, g, 1, counts, accumulate, nullptr, false, ws, stream));
}

int moe_predict_next(const moe_shape_t* shape, int32_t tokens, const void* x, const void* w_gate_next,
                     const float* gate_bias_next, int32_t* pred_idx, float* pred_w, int32_t* pred_counts,
                     void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (int rc = check_shape(shape)) return rc;
    if (tokens < 0 || tokens > kMaxTokens) return MOE_ERR_SHAPE;
    const void* const req[] = {w_gate_next, workspace};
    if (int rc = check_required(req)) return rc;
    const void* const per_token[] = {x, pred_idx};
    if (int rc = tokens > 0 ? check_required(per_token) : check_optional(per_token)) return rc;
    const void* const opt[] = {gate_bias_next, pred_w, pred_counts};
    if (int rc = check_optional(opt)) return rc;
    const WorkspaceLayout L = workspace_layout(*shape, tokens);
    if (workspace_bytes < L.route_end) return MOE_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const Ws ws = carve(workspace, L);
    if (tokens == 0) {
        if (pred_counts == nullptr) return MOE_OK;
        return dev(launch_finalize(*shape, 0, ws.hist, nullptr, pred_counts, 0, nullptr, nullptr, nullptr, nullptr, stream));
    }
    stage_call_begin(stream);
    GateArgs g[1] = {{w_gate_next, gate_bias_next, pred_idx, pred_w, nullptr}};
    return dev(run_route(*shape, tokens, x, g, 1, pred_counts, 0, nullptr, false, ws, stream));
}

int moe_expert_ffn(const moe_shape_t* shape, int32_t tokens, const void* x, const int32_t* topk_idx,
                   const float* topk_w, const void* w1, const void* w3, const void* w2, void* y, void* workspace,
                   size_t workspace_bytes, void* hip_stream) {
    if (int rc = check_shape(shape)) return rc;
    if (tokens < 0 || tokens > kMaxTokens) return MOE_ERR_SHAPE;
    const void* const req[] = {w1, w3, w2, workspace};
    if (int rc = check_required(req)) return rc;
    const void* const per_token[] = {x, topk_idx, topk_w, y};
    if (int rc = tokens > 0 ? check_required(per_token) : check_optional(per_token)) return rc;
    const WorkspaceLayout L = workspace_layout(*shape, tokens);
    if (workspace_bytes < L.total) return MOE_ERR_WORKSPACE;
    if (tokens == 0) return MOE_OK;
    return enqueue_expert_ffn(*shape, tokens, x, topk_idx, topk_w, w1, w3, w2, y, carve(workspace, L),
                              static_cast<hipStream_t>(hip_stream), kNoStaleInput);
}

int moe_expert_ffn_precalc(const moe_shape_t* shape, int32_t tokens, const void* x, const void* x_stale,
                           const uint8_t* stale, const int32_t* topk_idx, const float* topk_w, const void* w1,
                           const void* w3, const void* w2, void* y, void* workspace, size_t workspace_bytes,
                           void* hip_stream) {
    if (int rc = check_shape(shape)) return rc;
    if (tokens < 0 || tokens > kMaxTokens) return MOE_ERR_SHAPE;
    const void* const req[] = {w1, w3, w2, workspace};
    if (int rc = check_required(req)) return rc;
    const void* const per_token[] = {x, x_stale, stale, topk_idx, topk_w, y};
    if (int rc = tokens > 0 ? check_required(per_token) : check_optional(per_token)) return rc;
    const WorkspaceLayout L = workspace_layout(*shape, tokens);
    if (workspace_bytes < L.total) return MOE_ERR_WORKSPACE;
    if (tokens == 0) return MOE_OK;
    const StaleInput alt = {x_stale, stale};
    return enqueue_expert_ffn(*shape, tokens, x, topk_idx, topk_w, w1, w3, w2, y, carve(workspace, L),
                              static_cast<hipStream_t>(hip_stream), alt);
}

int moe_layer(const moe_shape_t* shape, int32_t tokens, const void* x, const void* w_gate, const float* gate_bias,
              const void* w_gate_next, const float* gate_bias_next, const void* w1, const void* w3, const void* w2,
              void* y, int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t accumulate, int32_t* pred_idx,
              void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (int rc = check_layer_args(shape, tokens, x, w_gate, gate_bias, w_gate_next, gate_bias_next, w1, w3, w2, y, topk_idx,
                                  topk_w, counts, pred_idx))
        return rc;
    const void* const req[] = {workspace};
    if (int rc = check_required(req)) return rc;
    const WorkspaceLayout L = workspace_layout(*shape, tokens);
    if (workspace_bytes < L.total) return MOE_ERR_WORKSPACE;
    return enqueue_layer(*shape, tokens, x, w_gate, gate_bias, w_gate_next, gate_bias_next, w1, w3, w2, y, topk_idx, topk_w,
                         counts, accumulate, pred_idx, carve(workspace, L), static_cast<hipStream_t>(hip_stream));
}

int moe_layer_static(const moe_shape_t* shape, int32_t tokens, const void* x, const void* w_gate,
                     const float* gate_bias, const void* w_gate_next, const float* gate_bias_next, const void* w1,
                     const void* w3, const void* w2, void* y, int32_t* topk_idx, float* topk_w, int32_t* counts,
                     int32_t accumulate, int32_t* pred_idx, void* hip_stream) {
    if (int rc = check_layer_args(shape, tokens, x, w_gate, gate_bias, w_gate_next, gate_bias_next, w1, w3, w2, y, topk_idx,
                                  topk_w, counts, pred_idx))
        return rc;
    const WorkspaceLayout L = workspace_layout(*shape, tokens);
    if (L.total > (size_t)MOE_STATIC_SCRATCH_BYTES) return MOE_ERR_TOO_LARGE;
    void* ws = static_scratch();
    if (ws == nullptr) return MOE_ERR_DEVICE;
    return enqueue_layer(*shape, tokens, x, w_gate, gate_bias, w_gate_next, gate_bias_next, w1, w3, w2, y, topk_idx, topk_w,
                         counts, accumulate, pred_idx, carve(ws, L), static_cast<hipStream_t>(hip_stream));
}

int moe_decode_status(void* workspace, size_t workspace_bytes, int32_t reset, int32_t* gave_up, void* hip_stream) {
    if (gave_up == nullptr) return MOE_ERR_NULL;
    if (workspace == nullptr) {  // the static scratch of moe_layer_static on the current device
        workspace = static_scratch();
        workspace_bytes = MOE_STATIC_SCRATCH_BYTES;
        if (workspace == nullptr) return MOE_ERR_DEVICE;
    }
    if (misaligned(workspace)) return MOE_ERR_ALIGN;
    if (workspace_bytes < kDecodeFlagInts * sizeof(uint32_t)) return MOE_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    uint32_t* word = static_cast<uint32_t*>(workspace) + kDecodeStatusWord;  // the flag block starts the workspace
    uint32_t value = 0;
    if (hipMemcpyAsync(&value, word, sizeof(value), hipMemcpyDeviceToHost, stream) != hipSuccess) return MOE_ERR_DEVICE;
    if (hipStreamSynchronize(stream) != hipSuccess) return MOE_ERR_DEVICE;
    *gave_up = value == kDecodeGaveUp ? 1 : 0;
    if (reset != 0) {
        const uint32_t zero = 0;
        if (hipMemcpyAsync(word, &zero, sizeof(zero), hipMemcpyHostToDevice, stream) != hipSuccess) return MOE_ERR_DEVICE;
        if (hipStreamSynchronize(stream) != hipSuccess) return MOE_ERR_DEVICE;
    }
    return MOE_OK;
}

int moe_measure_set_decode_spin_limit(int32_t polling_rounds) {
    if (polling_rounds < 0) return MOE_ERR_SHAPE;
    g_decode_spin_limit = polling_rounds;
    return MOE_OK;
}

int moe_stage_timing_begin(int32_t max_calls) {
    if (max_calls <= 0 || max_calls > 65536) return MOE_ERR_SHAPE;
    if (g_timer != nullptr) return MOE_ERR_SHAPE;
    StageTimer* t = new StageTimer();
    const int n = max_calls * StageTimer::kMaxMarks;
    t->max_calls = max_calls;
    t->events = new hipEvent_t[n];
    t->stage_of = new int[n];
    t->n_marks = new int[max_calls]();
    for (int i = 0; i < n; ++i) {
        if (hipEventCreate(&t->events[i]) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(t->events[j]);
            delete[] t->events; delete[] t->stage_of; delete[] t->n_marks; delete t;
            return MOE_ERR_DEVICE;
        }
    }
    g_timer = t;
    return MOE_OK;
}

int moe_stage_timing_end(float* stage_ms, int32_t* stage_launches) {
    StageTimer* t = g_timer;
    if (t == nullptr) return MOE_ERR_SHAPE;
    g_timer = nullptr;
    int rc = MOE_OK;
    double sum[MOE_NUM_STAGES] = {0};
    int cnt[MOE_NUM_STAGES] = {0};
    for (int c = 0; c < t->calls; ++c) {
        const int n = t->n_marks[c];
        hipEvent_t* ev = t->events + c * StageTimer::kMaxMarks;
        if (n > 0 && hipEventSynchronize(ev[n - 1]) != hipSuccess) rc = MOE_ERR_DEVICE;
        for (int i = 1; i < n; ++i) {
            float ms = 0.f;
            const int st = t->stage_of[c * StageTimer::kMaxMarks + i];
            if (hipEventElapsedTime(&ms, ev[i - 1], ev[i]) != hipSuccess) rc = MOE_ERR_DEVICE;
            else if (st >= 0 && st < MOE_NUM_STAGES) { sum[st] += ms; ++cnt[st]; }
        }
    }
    for (int s = 0; s < MOE_NUM_STAGES; ++s) {
        if (stage_ms != nullptr) stage_ms[s] = cnt[s] > 0 ? (float)(sum[s] / cnt[s]) : 0.f;
        if (stage_launches != nullptr) stage_launches[s] = cnt[s];
    }
    for (int i = 0; i < t->max_calls * StageTimer::kMaxMarks; ++i) (void)hipEventDestroy(t->events[i]);
    delete[] t->events; delete[] t->stage_of; delete[] t->n_marks; delete t;
    return rc;
}

}  // extern "C"
