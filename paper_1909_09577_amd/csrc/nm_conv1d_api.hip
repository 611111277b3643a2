// Host side of the C ABI declared in include/nm_conv1d.h: argument validation,
// choice between the matrix-core kernels and the plain kernels, workspace carving,
// launches.  Validation never touches the HIP runtime, so it behaves the same on a
// host without a device.
#include "../../include/nm_conv1d.h"
#include "nm_common.h"

#include <mutex>

using namespace nm;

// Scratch of nm_conv1d_block_fwd_static.  The name is a host-side handle only: device code and
// launches use the address hipGetSymbolAddress returns for the current device (static_scratch()).
static __device__ __align__(256) unsigned char scratch[NM_STATIC_SCRATCH_BYTES];

namespace {
// Address of `scratch` on the current device, looked up once per device.
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};
hipError_t static_scratch(void **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

thread_local hipEvent_t t_start_event = nullptr;
thread_local hipEvent_t t_stop_event = nullptr;
thread_local int t_timed_op = -1;    // pass whose main kernel the armed pair is for (-1: the first one launched)
thread_local int t_current_op = -1;  // pass the calling entry point is launching right now
}  // namespace

namespace nm {
DeviceInfo current_device_info()
{
    static int cached_cus[kMaxDevices] = {};  // 0: not asked yet
    DeviceInfo d = {-1, 256};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return d;
    d.dev = dev;
    if (dev < 0 || dev >= kMaxDevices) return d;
    if (cached_cus[dev] == 0) {
        int v = 0;
        cached_cus[dev] =
            (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) ? v : 256;
    }
    d.cus = cached_cus[dev];
    return d;
}

hipError_t ensure_dynamic_lds(LdsOptIn &state, const void *fn, int bytes)
{
    const DeviceInfo d = current_device_info();
    const bool known = d.dev >= 0 && d.dev < kMaxDevices;
    if (known && state.done[d.dev]) return hipSuccess;
    const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && known) state.done[d.dev] = 1;
    return e;
}

MainKernelTimer::MainKernelTimer(hipStream_t s) : stream(s), stop(nullptr)
{
    if (!(t_start_event && t_stop_event)) return;
    if (t_timed_op >= 0 && t_timed_op != t_current_op) return;  // armed for another pass of this call
    (void)hipEventRecord(t_start_event, s);
    stop = t_stop_event;
    t_start_event = nullptr;
    t_stop_event = nullptr;
}
MainKernelTimer::~MainKernelTimer()
{
    if (stop) (void)hipEventRecord(stop, stream);
}
}  // namespace nm

namespace {

constexpr unsigned kAllFlags = NM_RELU | NM_ACCUM_DW | NM_FORCE_DIRECT | NM_ACCUM_DX;
constexpr size_t kWsAlign = 256;
constexpr long long kMaxElems = (1LL << 31) - 1;

int out_len(int T, int K, int stride, int dil, int pad)
{
    if (T <= 0 || K <= 0 || stride <= 0 || dil <= 0 || pad < 0) return NM_ERR_BAD_ARG;
    const long long span = (long long)T + 2LL * pad - (long long)dil * (K - 1) - 1;
    if (span < 0) return NM_ERR_BAD_ARG;
    const long long to = span / stride + 1;
    if (to > kMaxElems) return NM_ERR_BAD_ARG;
    return (int)to;
}

// Fills g; returns NM_OK or the status to hand back.
int check_geometry(int B, int Cin, int Cout, int T, int K, int stride, int dil, int pad, int dtype,
                   unsigned flags, unsigned allowed_flags, Geom *g)
{
    if (B <= 0 || Cin <= 0 || Cout <= 0) return NM_ERR_BAD_ARG;
    const int to = out_len(T, K, stride, dil, pad);
    if (to <= 0) return NM_ERR_BAD_ARG;
    if (dtype != NM_BF16 && dtype != NM_F32) return NM_ERR_BAD_ARG;
    if (flags & ~allowed_flags) return NM_ERR_BAD_ARG;
    if ((long long)B * Cin * T > kMaxElems || (long long)B * Cout * to > kMaxElems ||
        (long long)Cout * Cin * K > kMaxElems)
        return NM_ERR_UNSUPPORTED;
    if (B > 65535 || Cout > 65535 || Cin > 65535) return NM_ERR_UNSUPPORTED;  // grid y/z limits
    if ((long long)pad + (long long)dil * K > (1 << 28) || stride > (1 << 20)) return NM_ERR_UNSUPPORTED;
    g->B = B; g->Cin = Cin; g->Cout = Cout; g->T = T; g->K = K;
    g->stride = stride; g->dil = dil; g->pad = pad; g->To = to;
    g->len = nullptr;
    return NM_OK;
}

bool overlap(const void *a, size_t na, const void *b, size_t nb)
{
    if (!a || !b) return false;
    const char *pa = (const char *)a, *pb = (const char *)b;
    return pa < pb + nb && pb < pa + na;
}

size_t elt(int dtype) { return dtype == NM_BF16 ? 2 : 4; }

bool use_mfma(int op, const Geom &g, int dtype, unsigned flags)
{
    if (dtype != NM_BF16 || (flags & NM_FORCE_DIRECT)) return false;
    switch (op) {
    case NM_OP_FWD: return mfma_fwd_supported(g);
    case NM_OP_BWD_DATA: return mfma_dgrad_supported(g);
    case NM_OP_BWD_WEIGHT: return mfma_wgrad_supported(g);
    default: return false;
    }
}

// Whether dz = dy*[y>0]*scale differs from dy (the plain input-gradient kernel contracts a materialised dz;
// the plain weight-gradient kernel contracts dy*[y>0] and applies scale to its sums).
bool needs_dz(unsigned flags, const float *scale) { return (flags & NM_RELU) || scale != nullptr; }

bool aligned16(const void *p) { return ((uintptr_t)p % 16) == 0; }

// Whether a call with per-sample lengths may take the matrix-core kernels: the forward pass, the input
// gradient and the stride-1 weight-gradient kernels apply them; the general weight-gradient kernel
// does not (lengths then go to the plain kernel).
bool masked_on_mfma(const Geom &g, int op = NM_OP_FWD)
{
    return g.len == nullptr || op != NM_OP_BWD_WEIGHT || mfma_wgrad_fast_supported(g);
}

// Scratch need of one operation on one path (mfma: matrix-core kernels, else plain kernels).
size_t workspace_for(int op, const Geom &g, int dtype, bool mfma, bool scale_or_relu)
{
    if (mfma) {
        if (op == NM_OP_FWD) return mfma_fwd_workspace(g);
        if (op == NM_OP_BWD_DATA) return mfma_dgrad_workspace(g);
        return mfma_wgrad_workspace(g, scale_or_relu);
    }
    if (op == NM_OP_FWD) return 0;
    return scale_or_relu ? align_up((size_t)g.B * g.Cout * g.To * elt(dtype), kWsAlign) : 0;
}

int check_workspace(const void *ws, size_t have, size_t need)
{
    if (need == 0) return NM_OK;
    if (!ws || have < need || ((uintptr_t)ws % kWsAlign) != 0) return NM_ERR_WORKSPACE;
    return NM_OK;
}

int dev(hipError_t e) { return e == hipSuccess ? NM_OK : NM_ERR_DEVICE; }

// Consumes the armed event pair when an entry point returns without launching its main kernel.
struct DisarmOnExit {
    ~DisarmOnExit()
    {
        t_start_event = nullptr;
        t_stop_event = nullptr;
        t_current_op = -1;
    }
};

}  // namespace

extern "C" {

int nm_conv1d_out_len(int T, int K, int stride, int dilation, int pad)
{
    return out_len(T, K, stride, dilation, pad);
}

size_t nm_conv1d_workspace_bytes(int op, int B, int Cin, int Cout, int T, int K, int stride, int dilation,
                                 int pad, int dtype, unsigned flags)
{
    Geom g;
    if (op != NM_OP_FWD && op != NM_OP_BWD_DATA && op != NM_OP_BWD_WEIGHT && op != NM_OP_BWD && op != NM_OP_BN_FWD &&
        op != NM_OP_BN_BWD)
        return 0;
    if (check_geometry(B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags, kAllFlags, &g) != NM_OK)
        return 0;
    // the BatchNorm calls keep their own scratch (and, backward, the dz tensor) in front of the inner call's workspace
    if (op == NM_OP_BN_FWD)
        return bn_fwd_scratch_bytes(g.B, g.Cout, g.To) +
               nm_conv1d_workspace_bytes(NM_OP_FWD, B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags);
    if (op == NM_OP_BN_BWD)
        return bn_bwd_scratch_bytes(g.B, g.Cout) + align_up((size_t)g.B * g.Cout * g.To * elt(dtype), kWsAlign) +
               nm_conv1d_workspace_bytes(NM_OP_BWD, B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags);
    // The query sees neither the scale pointer nor the alignment of the tensors (misaligned
    // tensors take the plain kernels); it sizes for the larger of the cases.
    auto one = [&](int o) {
        const size_t plain = workspace_for(o, g, dtype, false, true);
        const size_t fast = use_mfma(o, g, dtype, flags) ? workspace_for(o, g, dtype, true, true) : 0;
        return plain > fast ? plain : fast;
    };
    // the fused backward keeps the two gradients' workspaces side by side
    if (op == NM_OP_BWD) return one(NM_OP_BWD_DATA) + one(NM_OP_BWD_WEIGHT);
    return one(op);
}

int nm_conv1d_time_next_main_kernel(void *start_event, void *stop_event)
{
    t_start_event = (start_event && stop_event) ? (hipEvent_t)start_event : nullptr;
    t_stop_event = (start_event && stop_event) ? (hipEvent_t)stop_event : nullptr;
    t_timed_op = -1;
    return NM_OK;
}

int nm_conv1d_time_next_kernel_of(void *start_event, void *stop_event, int op)
{
    if (op != NM_OP_FWD && op != NM_OP_BWD_DATA && op != NM_OP_BWD_WEIGHT) return NM_ERR_BAD_ARG;
    nm_conv1d_time_next_main_kernel(start_event, stop_event);
    t_timed_op = op;
    return NM_OK;
}

const char *nm_strerror(int status)
{
    switch (status) {
    case NM_OK: return "ok";
    case NM_ERR_BAD_ARG: return "invalid argument";
    case NM_ERR_UNSUPPORTED: return "unsupported size";
    case NM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case NM_ERR_DEVICE: return "HIP runtime error";
    case NM_ERR_SCRATCH_LIMIT: return "geometry needs more scratch than the fixed array of the no-allocation entry point";
    default: return "unknown status";
    }
}

static int block_fwd_impl(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const int *lengths,
                          const void *x, const void *w, const float *scale, const float *shift,
                          const void *residual, void *y, unsigned flags, int dtype, void *workspace,
                          size_t workspace_bytes, void *hip_stream, double *stats = nullptr, int *stats_parts = nullptr)
{
    // stats / stats_parts (the BatchNorm entry point): where the kernel that runs can write the partial statistics of
    // its outputs it does, and *stats_parts says into how many parts per channel (0: it did not)
    DisarmOnExit disarm;
    if (stats_parts) *stats_parts = 0;
    Geom g;
    int st = check_geometry(B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags,
                            NM_RELU | NM_FORCE_DIRECT, &g);
    if (st != NM_OK) return st;
    if (!x || !w || !y) return NM_ERR_BAD_ARG;
    g.len = lengths;
    const size_t e = elt(dtype);
    const size_t ny = (size_t)g.B * g.Cout * g.To * e;
    if (overlap(y, ny, x, (size_t)g.B * g.Cin * g.T * e) || overlap(y, ny, w, (size_t)g.Cout * g.Cin * g.K * e) ||
        overlap(y, ny, residual, ny))
        return NM_ERR_BAD_ARG;
    const bool mfma = use_mfma(NM_OP_FWD, g, dtype, flags) && aligned16(x) && aligned16(y) && aligned16(residual) &&
                      masked_on_mfma(g);
    const size_t need = workspace_for(NM_OP_FWD, g, dtype, mfma, true);
    st = check_workspace(workspace, workspace_bytes, need);
    if (st != NM_OK) return st;
    if (overlap(y, ny, workspace, need)) return NM_ERR_BAD_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    const bool relu = (flags & NM_RELU) != 0;
    t_current_op = NM_OP_FWD;
    if (mfma) {
        const int parts = (stats && stats_parts) ? mfma_fwd_stats_parts(g) : 0;
        const hipError_t err = launch_mfma_fwd(g, x, w, scale, shift, residual, y, relu, workspace, s, parts > 0 ? stats : nullptr);
        if (err == hipSuccess && parts > 0) *stats_parts = parts;
        return dev(err);
    }
    MainKernelTimer timer(s);
    return dev(launch_direct_fwd(g, dtype == NM_BF16, x, w, scale, shift, residual, y, relu, s));
}

static int bwd_data_impl(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const int *lengths,
                         const void *dy, const void *y, const float *scale, const void *w, void *dx,
                         void *dres, unsigned flags, int dtype, void *workspace, size_t workspace_bytes,
                         void *hip_stream)
{
    DisarmOnExit disarm;
    Geom g;
    int st = check_geometry(B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags,
                            NM_RELU | NM_FORCE_DIRECT | NM_ACCUM_DX, &g);
    if (st != NM_OK) return st;
    if (!dy || !w || !dx) return NM_ERR_BAD_ARG;
    g.len = lengths;
    const bool relu = (flags & NM_RELU) != 0;
    if (relu && !y) return NM_ERR_BAD_ARG;
    const size_t e = elt(dtype);
    const size_t ndy = (size_t)g.B * g.Cout * g.To * e, ndx = (size_t)g.B * g.Cin * g.T * e;
    if (overlap(dx, ndx, dy, ndy) || overlap(dx, ndx, y, ndy) || overlap(dx, ndx, w, (size_t)g.Cout * g.Cin * g.K * e) ||
        overlap(dx, ndx, dres, ndy) || overlap(dres, ndy, dy, ndy) || overlap(dres, ndy, y, ndy))
        return NM_ERR_BAD_ARG;
    const bool accum = (flags & NM_ACCUM_DX) != 0;
    // accumulation into dx: the matrix-core engine adds the old value in its epilogue (stride 1, no lengths)
    const bool mfma = use_mfma(NM_OP_BWD_DATA, g, dtype, flags) && aligned16(dy) && aligned16(dx) &&
                      (!relu || aligned16(y)) && masked_on_mfma(g) && !(accum && (g.stride != 1 || g.len));
    const bool dzneeded = needs_dz(flags, scale);
    const size_t need = workspace_for(NM_OP_BWD_DATA, g, dtype, mfma, dzneeded);
    st = check_workspace(workspace, workspace_bytes, need);
    if (st != NM_OK) return st;
    if (overlap(dx, ndx, workspace, need) || overlap(dres, ndy, workspace, need)) return NM_ERR_BAD_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    t_current_op = NM_OP_BWD_DATA;
    if (mfma) return dev(launch_mfma_dgrad(g, dy, y, scale, w, dx, dres, relu, accum, workspace, s));
    const bool bf = dtype == NM_BF16;
    const void *dz = dy;
    if (dzneeded || dres) {
        hipError_t err = launch_epilogue_bwd(g, bf, dy, y, scale, relu, dzneeded ? workspace : nullptr, dres, s);
        if (err != hipSuccess) return NM_ERR_DEVICE;
        if (dzneeded) dz = workspace;
    }
    MainKernelTimer timer(s);
    return dev(launch_direct_dgrad(g, bf, dz, w, dx, accum, s));
}

static int bwd_weight_impl(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const int *lengths,
                           const void *x, const void *dy, const void *y, const float *scale, float *dw,
                           unsigned flags, int dtype, void *workspace, size_t workspace_bytes,
                           void *hip_stream)
{
    DisarmOnExit disarm;
    Geom g;
    int st = check_geometry(B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags,
                            NM_RELU | NM_ACCUM_DW | NM_FORCE_DIRECT, &g);
    if (st != NM_OK) return st;
    if (!x || !dy || !dw) return NM_ERR_BAD_ARG;
    g.len = lengths;
    const bool relu = (flags & NM_RELU) != 0;
    if (relu && !y) return NM_ERR_BAD_ARG;
    const size_t e = elt(dtype);
    const size_t ndy = (size_t)g.B * g.Cout * g.To * e, ndw = (size_t)g.Cout * g.Cin * g.K * sizeof(float);
    if (overlap(dw, ndw, dy, ndy) || overlap(dw, ndw, y, ndy) || overlap(dw, ndw, x, (size_t)g.B * g.Cin * g.T * e))
        return NM_ERR_BAD_ARG;
    const bool mfma = use_mfma(NM_OP_BWD_WEIGHT, g, dtype, flags) && aligned16(x) && aligned16(dy) &&
                      (!relu || aligned16(y)) && masked_on_mfma(g, NM_OP_BWD_WEIGHT);
    const bool dzneeded = needs_dz(flags, scale);
    const size_t need = workspace_for(NM_OP_BWD_WEIGHT, g, dtype, mfma, dzneeded);
    st = check_workspace(workspace, workspace_bytes, need);
    if (st != NM_OK) return st;
    if (overlap(dw, ndw, workspace, need)) return NM_ERR_BAD_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    const bool accum = (flags & NM_ACCUM_DW) != 0;
    t_current_op = NM_OP_BWD_WEIGHT;
    if (mfma) return dev(launch_mfma_wgrad(g, x, dy, y, scale, dw, relu, accum, workspace, s));
    const bool bf = dtype == NM_BF16;
    const void *dz = dy;
    if (relu) {  // the kernel contracts dy*[y>0]; scale multiplies its float32 sums
        hipError_t err = launch_epilogue_bwd(g, bf, dy, y, nullptr, relu, workspace, nullptr, s);
        if (err != hipSuccess) return NM_ERR_DEVICE;
        dz = workspace;
    }
    MainKernelTimer timer(s);
    return dev(launch_direct_wgrad(g, bf, x, dz, scale, dw, accum, s));
}

int nm_conv1d_block_fwd(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const void *x,
                        const void *w, const float *scale, const float *shift, const void *residual, void *y,
                        unsigned flags, int dtype, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return block_fwd_impl(B, Cin, Cout, T, K, stride, dilation, pad, nullptr, x, w, scale, shift, residual, y, flags, dtype,
                          workspace, workspace_bytes, hip_stream);
}

int nm_conv1d_block_fwd_static(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const void *x,
                               const void *w, const float *scale, const float *shift, const void *residual, void *y,
                               unsigned flags, int dtype, void *hip_stream)
{
    // Size the scratch like nm_conv1d_workspace_bytes does (0 for invalid arguments: the shared
    // implementation below then reports them, before any device call).
    const size_t need = nm_conv1d_workspace_bytes(NM_OP_FWD, B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags);
    if (need > NM_STATIC_SCRATCH_BYTES) {
        DisarmOnExit disarm;
        return NM_ERR_SCRATCH_LIMIT;
    }
    void *ptr = nullptr;
    if (need > 0 && x && w && y) {  // (missing tensors: no device call before the argument error)
        if (static_scratch(&ptr) != hipSuccess) {
            DisarmOnExit disarm;
            return NM_ERR_DEVICE;
        }
    }
    return block_fwd_impl(B, Cin, Cout, T, K, stride, dilation, pad, nullptr, x, w, scale, shift, residual, y, flags, dtype,
                          ptr, ptr ? (size_t)NM_STATIC_SCRATCH_BYTES : 0, hip_stream);
}

int nm_conv1d_bwd_data(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const void *dy,
                       const void *y, const float *scale, const void *w, void *dx, void *dres, unsigned flags, int dtype,
                       void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return bwd_data_impl(B, Cin, Cout, T, K, stride, dilation, pad, nullptr, dy, y, scale, w, dx, dres, flags, dtype,
                         workspace, workspace_bytes, hip_stream);
}

int nm_conv1d_bwd_weight(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const void *x,
                         const void *dy, const void *y, const float *scale, float *dw, unsigned flags, int dtype,
                         void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return bwd_weight_impl(B, Cin, Cout, T, K, stride, dilation, pad, nullptr, x, dy, y, scale, dw, flags, dtype, workspace,
                           workspace_bytes, hip_stream);
}

int nm_conv1d_block_fwd_masked(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                               const int *lengths, const void *x, const void *w, const float *scale, const float *shift,
                               const void *residual, void *y, unsigned flags, int dtype, void *workspace,
                               size_t workspace_bytes, void *hip_stream)
{
    if (!lengths) return NM_ERR_BAD_ARG;
    return block_fwd_impl(B, Cin, Cout, T, K, stride, dilation, pad, lengths, x, w, scale, shift, residual, y, flags, dtype,
                          workspace, workspace_bytes, hip_stream);
}

int nm_conv1d_bwd_data_masked(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                              const int *lengths, const void *dy, const void *y, const float *scale, const void *w,
                              void *dx, void *dres, unsigned flags, int dtype, void *workspace, size_t workspace_bytes,
                              void *hip_stream)
{
    if (!lengths) return NM_ERR_BAD_ARG;
    return bwd_data_impl(B, Cin, Cout, T, K, stride, dilation, pad, lengths, dy, y, scale, w, dx, dres, flags, dtype,
                         workspace, workspace_bytes, hip_stream);
}

int nm_conv1d_bwd_weight_masked(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad,
                                const int *lengths, const void *x, const void *dy, const void *y, const float *scale,
                                float *dw, unsigned flags, int dtype, void *workspace, size_t workspace_bytes,
                                void *hip_stream)
{
    if (!lengths) return NM_ERR_BAD_ARG;
    return bwd_weight_impl(B, Cin, Cout, T, K, stride, dilation, pad, lengths, x, dy, y, scale, dw, flags, dtype, workspace,
                           workspace_bytes, hip_stream);
}

static int bwd_impl(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const int *lengths,
                    const void *x, const void *dy, const void *y, const float *scale, const void *w, void *dx, void *dres,
                    float *dw, unsigned flags, int dtype, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Geom g;
    int st = check_geometry(B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags, kAllFlags, &g);
    if (st == NM_OK && (!x || !dy || !w || !dx || !dw)) st = NM_ERR_BAD_ARG;
    if (st == NM_OK && (flags & NM_RELU) && !y) st = NM_ERR_BAD_ARG;
    const size_t need =
        st == NM_OK ? nm_conv1d_workspace_bytes(NM_OP_BWD, B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags) : 0;
    if (st == NM_OK) st = check_workspace(workspace, workspace_bytes, need);
    if (st != NM_OK) {
        DisarmOnExit disarm;  // an armed timer is consumed by this call whatever happens
        return st;
    }
    const bool relu = (flags & NM_RELU) != 0;
    g.len = lengths;
    const bool fused = !(lengths && (flags & NM_ACCUM_DX)) &&
                       use_mfma(NM_OP_BWD_DATA, g, dtype, flags) && use_mfma(NM_OP_BWD_WEIGHT, g, dtype, flags) &&
                       g.stride == 1 && mfma_wgrad_fast_supported(g) && !wgrad_k1_supported(g) && aligned16(x) && aligned16(dy) &&
                       aligned16(dx) && (!relu || aligned16(y)) && (!dres || aligned16(dres));
    const size_t ws_data = mfma_dgrad_workspace(g);  // only meaningful when fused
    // pointwise layers: the input gradient's masked g = dy*[y>0] also feeds the K=1 weight-gradient GEMM
    const bool fused_k1 = !lengths && g.stride == 1 && use_mfma(NM_OP_BWD_DATA, g, dtype, flags) &&
                          use_mfma(NM_OP_BWD_WEIGHT, g, dtype, flags) && wgrad_k1_supported(g) && aligned16(x) &&
                          aligned16(dy) && aligned16(dx) && (!relu || aligned16(y));
    if (fused_k1) {
        DisarmOnExit disarm;
        const size_t e = elt(dtype);
        const size_t ndy = (size_t)g.B * g.Cout * g.To * e, nx = (size_t)g.B * g.Cin * g.T * e;
        const size_t nw = (size_t)g.Cout * g.Cin * g.K * e, ndw = (size_t)g.Cout * g.Cin * g.K * sizeof(float);
        if (overlap(dx, nx, dy, ndy) || overlap(dx, nx, y, ndy) || overlap(dx, nx, w, nw) || overlap(dx, nx, x, nx) ||
            overlap(dres, ndy, dy, ndy) || overlap(dres, ndy, y, ndy) || overlap(dres, ndy, dx, nx) ||
            overlap(dw, ndw, dy, ndy) || overlap(dw, ndw, y, ndy) || overlap(dw, ndw, x, nx) || overlap(dw, ndw, dx, nx) ||
            overlap(dw, ndw, dres, ndy) || overlap(dx, nx, workspace, need) || overlap(dres, ndy, workspace, need) ||
            overlap(dw, ndw, workspace, need))
            return NM_ERR_BAD_ARG;
        hipStream_t s = (hipStream_t)hip_stream;
        const void *g_plain = nullptr;
        t_current_op = NM_OP_BWD_DATA;
        hipError_t err = launch_mfma_dgrad(g, dy, y, scale, w, dx, dres, relu, (flags & NM_ACCUM_DX) != 0, workspace, s, &g_plain);
        if (err != hipSuccess || !g_plain) return NM_ERR_DEVICE;
        t_current_op = NM_OP_BWD_WEIGHT;
        return dev(launch_wgrad_k1(g, x, g_plain, scale, dw, (flags & NM_ACCUM_DW) != 0, (unsigned char *)workspace + ws_data, s));
    }
    if (!fused) {
        // two calls sharing the workspace one after the other (their own argument checks apply)
        const size_t w1 = nm_conv1d_workspace_bytes(NM_OP_BWD_DATA, B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags);
        // a timer armed for the weight-gradient kernel outlives the first of the two calls
        hipEvent_t keep_start = t_start_event, keep_stop = t_stop_event;
        const bool keep = t_timed_op == NM_OP_BWD_WEIGHT;
        st = bwd_data_impl(B, Cin, Cout, T, K, stride, dilation, pad, lengths, dy, y, scale, w, dx, dres, flags & ~NM_ACCUM_DW,
                           dtype, workspace, w1, hip_stream);
        if (st != NM_OK) return st;
        if (keep) {
            t_start_event = keep_start;
            t_stop_event = keep_stop;
        }
        return bwd_weight_impl(B, Cin, Cout, T, K, stride, dilation, pad, lengths, x, dy, y, scale, dw, flags & ~NM_ACCUM_DX,
                               dtype, workspace, workspace_bytes, hip_stream);
    }
    DisarmOnExit disarm;
    const size_t e = elt(dtype);
    const size_t ndy = (size_t)g.B * g.Cout * g.To * e, nx = (size_t)g.B * g.Cin * g.T * e;
    const size_t nw = (size_t)g.Cout * g.Cin * g.K * e, ndw = (size_t)g.Cout * g.Cin * g.K * sizeof(float);
    if (overlap(dx, nx, dy, ndy) || overlap(dx, nx, y, ndy) || overlap(dx, nx, w, nw) || overlap(dx, nx, x, nx) ||
        overlap(dres, ndy, dy, ndy) || overlap(dres, ndy, y, ndy) || overlap(dres, ndy, dx, nx) ||
        overlap(dw, ndw, dy, ndy) || overlap(dw, ndw, y, ndy) || overlap(dw, ndw, x, nx) || overlap(dw, ndw, dx, nx) ||
        overlap(dw, ndw, dres, ndy) || overlap(dx, nx, workspace, need) || overlap(dres, ndy, workspace, need) ||
        overlap(dw, ndw, workspace, need))
        return NM_ERR_BAD_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    void *ws_w = (unsigned char *)workspace + ws_data;  // the weight gradient's workspace: partials, then dz fragments
    const DzfLayout layout = mfma_wgrad_dzf_layout(g);
    const void *g_plain = nullptr;
    hipError_t err = launch_bwd_prepare(g, dy, y, scale, w, relu, workspace, (unsigned char *)ws_w + layout.offset, layout,
                                        dres, &g_plain, s);
    if (err != hipSuccess) return NM_ERR_DEVICE;
    t_current_op = NM_OP_BWD_DATA;
    err = launch_mfma_dgrad_prepared(g, g_plain, dx, (flags & NM_ACCUM_DX) != 0, workspace, s);
    if (err != hipSuccess) return NM_ERR_DEVICE;
    t_current_op = NM_OP_BWD_WEIGHT;
    return dev(launch_mfma_wgrad_prepared(g, x, scale, dw, (flags & NM_ACCUM_DW) != 0, ws_w, s));
}

int nm_conv1d_bwd(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const void *x,
                  const void *dy, const void *y, const float *scale, const void *w, void *dx, void *dres, float *dw,
                  unsigned flags, int dtype, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return bwd_impl(B, Cin, Cout, T, K, stride, dilation, pad, nullptr, x, dy, y, scale, w, dx, dres, dw, flags, dtype,
                    workspace, workspace_bytes, hip_stream);
}

int nm_conv1d_bwd_masked(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const int *lengths,
                         const void *x, const void *dy, const void *y, const float *scale, const void *w, void *dx,
                         void *dres, float *dw, unsigned flags, int dtype, void *workspace, size_t workspace_bytes,
                         void *hip_stream)
{
    if (!lengths) return NM_ERR_BAD_ARG;
    return bwd_impl(B, Cin, Cout, T, K, stride, dilation, pad, lengths, x, dy, y, scale, w, dx, dres, dw, flags, dtype,
                    workspace, workspace_bytes, hip_stream);
}

int nm_conv1d_bn_fwd(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const void *x,
                     const void *w, const float *gamma, const float *beta, float eps, const void *residual, void *z,
                     void *y, float *mean, float *invstd, unsigned flags, int dtype, void *workspace,
                     size_t workspace_bytes, void *hip_stream)
{
    Geom g;
    int st = check_geometry(B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags, NM_RELU | NM_FORCE_DIRECT, &g);
    if (st == NM_OK && (!x || !w || !z || !y || !mean || !invstd || !(eps >= 0.f))) st = NM_ERR_BAD_ARG;
    const size_t e = st == NM_OK ? elt(dtype) : 0;
    const size_t ny = st == NM_OK ? (size_t)g.B * g.Cout * g.To * e : 0;
    if (st == NM_OK && (overlap(y, ny, z, ny) || overlap(y, ny, residual, ny) || overlap(z, ny, residual, ny) ||
                        overlap(y, ny, x, (size_t)g.B * g.Cin * g.T * e) || overlap(y, ny, w, (size_t)g.Cout * g.Cin * g.K * e)))
        st = NM_ERR_BAD_ARG;
    const size_t need =
        st == NM_OK ? nm_conv1d_workspace_bytes(NM_OP_BN_FWD, B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags) : 0;
    if (st == NM_OK) st = check_workspace(workspace, workspace_bytes, need);
    if (st == NM_OK && (overlap(y, ny, workspace, need) || overlap(z, ny, workspace, need))) st = NM_ERR_BAD_ARG;
    if (st != NM_OK) {
        DisarmOnExit disarm;
        return st;
    }
    const size_t own = bn_fwd_scratch_bytes(g.B, g.Cout, g.To);
    // the convolution itself: z = conv(x, w), no epilogue (its own argument checks apply once more); the unrolled
    // matrix-core kernels write the partial statistics of z from their epilogue, for the others a pass over z follows
    int parts = 0;
    st = block_fwd_impl(B, Cin, Cout, T, K, stride, dilation, pad, nullptr, x, w, nullptr, nullptr, nullptr, z,
                        flags & NM_FORCE_DIRECT, dtype, (unsigned char *)workspace + own, workspace_bytes - own, hip_stream,
                        (double *)workspace, &parts);
    if (st != NM_OK) return st;
    return dev(launch_bn_fwd(g.B, g.Cout, g.To, dtype == NM_BF16, z, gamma, beta, eps, residual, (flags & NM_RELU) != 0, y, mean,
                             invstd, workspace, (hipStream_t)hip_stream, parts));
}

int nm_conv1d_bn_bwd(int B, int Cin, int Cout, int T, int K, int stride, int dilation, int pad, const void *x,
                     const void *w, const float *gamma, const void *z, const void *y, const float *mean,
                     const float *invstd, const void *dy, void *dx, void *dres, float *dw, float *dgamma, float *dbeta,
                     unsigned flags, int dtype, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Geom g;
    int st = check_geometry(B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags, kAllFlags, &g);
    if (st == NM_OK && (!x || !w || !z || !mean || !invstd || !dy || !dx || !dw)) st = NM_ERR_BAD_ARG;
    if (st == NM_OK && (flags & NM_RELU) && !y) st = NM_ERR_BAD_ARG;
    const size_t e = st == NM_OK ? elt(dtype) : 0;
    const size_t ny = st == NM_OK ? (size_t)g.B * g.Cout * g.To * e : 0;
    if (st == NM_OK && (overlap(dres, ny, dy, ny) || overlap(dres, ny, y, ny) || overlap(dres, ny, z, ny))) st = NM_ERR_BAD_ARG;
    const size_t need =
        st == NM_OK ? nm_conv1d_workspace_bytes(NM_OP_BN_BWD, B, Cin, Cout, T, K, stride, dilation, pad, dtype, flags) : 0;
    if (st == NM_OK) st = check_workspace(workspace, workspace_bytes, need);
    if (st == NM_OK && overlap(dres, ny, workspace, need)) st = NM_ERR_BAD_ARG;
    if (st != NM_OK) {
        DisarmOnExit disarm;
        return st;
    }
    const size_t own = bn_bwd_scratch_bytes(g.B, g.Cout);
    void *dz = (unsigned char *)workspace + own;
    const size_t used = own + align_up(ny, kWsAlign);
    const bool relu = (flags & NM_RELU) != 0;
    hipError_t err = launch_bn_bwd(g.B, g.Cout, g.To, dtype == NM_BF16, dy, y, z, gamma, mean, invstd, relu, dz, dres, dgamma,
                                   dbeta, (flags & NM_ACCUM_DW) != 0, workspace, (hipStream_t)hip_stream);
    if (err != hipSuccess) {
        DisarmOnExit disarm;
        return NM_ERR_DEVICE;
    }
    // both convolution gradients of the corrected dz (no mask, no scale left to apply)
    return nm_conv1d_bwd(B, Cin, Cout, T, K, stride, dilation, pad, x, dz, nullptr, nullptr, w, dx, nullptr, dw,
                         flags & (NM_ACCUM_DW | NM_ACCUM_DX | NM_FORCE_DIRECT), dtype, (unsigned char *)workspace + used,
                         workspace_bytes - used, hip_stream);
}

}  // extern "C"
