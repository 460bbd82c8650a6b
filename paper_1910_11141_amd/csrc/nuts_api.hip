// Host side of the C ABI declared in include/nuts.h: argument validation,
// target construction (device copies in kernel-friendly layouts), workspace
// management, kernel selection and launch.  There is no CPU fallback: if the
// device is missing or a launch fails the call returns NUTS_E_DEVICE.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/nuts.h"
#include "nuts_dev.h"
#include "nuts_dense.h"
#include "nuts_elem.h"
#include "nuts_grid.h"
#include "nuts_quad.h"
#include "nuts_tile.h"
#include "nuts_wave.h"

namespace {

thread_local char g_err[512] = "";
thread_local hipStream_t g_stream = nullptr;

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr, code)                                                                      \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess) return fail((code), "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

size_t elem_size(int dtype) { return dtype == NUTS_F64 ? sizeof(double) : sizeof(float); }

// Scratch memory of nuts_sample_static: one array per GPU, part of the loaded code object, never
// allocated or freed.  The first kStaticHeader bytes hold the call's counters, the rest its workspace.
// In host code the array's name is only a handle for hipGetSymbolAddress; kernels get the address that
// call returned for the current device.
constexpr size_t kStaticHeader = 256;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[NUTS_STATIC_SCRATCH_BYTES];
unsigned char* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, looked up once
std::mutex g_scratch_mutex;

// Looks up the current device's copy of `scratch` (set-up time: target creation or a first regular call).
int resolve_scratch(int dev)
{
    if (dev < 0 || dev >= kMaxDevices) return fail(NUTS_E_UNSUPPORTED, "device index %d out of range", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), NUTS_E_DEVICE);
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    return NUTS_OK;
}

}  // namespace

struct nuts_target {
    int32_t kind = 0, dtype = 0;
    int64_t dim = 0, n = 0;
    double prior_scale = 1.0;
    int device = -1;  // -1: no device data (standard normal before its first use)
    // device copies
    void* dPT = nullptr;
    void* dFtab = nullptr;  // table of the logistic function for the weight merges of the register kernels
    void* dBand = nullptr;  // banded precision matrices of dim <= kBandRows: the band, see DevTarget::band
    void* dInvVar = nullptr;
    void* dX = nullptr;
    void* dXT = nullptr;
    void* dY = nullptr;
    nuts::TileData tile;  // operand-order copies of X for the tile kernel (binary64 logistic regression)
    nuts::GridData grid;  // operand-order copy of X for the grid kernels (binary32 logistic regression)
    nuts::QuadData quad;  // operand-order copy of P for the quad kernel (binary64 dense Gaussian, dim <= 128)
    // per-call scratch, grown on demand and kept
    char* workspace = nullptr;
    size_t workspace_bytes = 0;
    unsigned long long* counters = nullptr;
    // where the call in progress keeps its workspace and counters: the target's own allocations, or the
    // device's static scratch array (nuts_sample_static)
    bool static_call = false;
    char* ws_cur = nullptr;
    unsigned long long* counters_cur = nullptr;
    hipEvent_t ev_start = nullptr, ev_stop = nullptr;
    // grid kernels: the sets of chains beyond the first run their rounds on these streams
    hipStream_t side_stream[nuts::kGridMaxStreams - 1] = {};
    hipEvent_t ev_fork = nullptr, ev_join[nuts::kGridMaxStreams - 1] = {};
    int* halted_host = nullptr;         // grid kernels: pinned, two snapshots of the "halted" flags
    hipEvent_t ev_batch[2 * nuts::kGridMaxStreams] = {};  // [snapshot][stream]
    bool has_run = false;
    int32_t last_variant = 0, last_grid = 0;
    long last_slots = 0;       // chain slots of the last launch if the host charges them (wave, element-wise), else 0
    void* carry = nullptr;     // states handed from launch to launch under the trajectory schedule
    size_t carry_bytes = 0;
};

namespace {

template <typename T>
int upload(const std::vector<T>& host, void** dev)
{
    HIP_TRY(hipMalloc(dev, host.size() * sizeof(T)), NUTS_E_ALLOC);
    HIP_TRY(hipMemcpy(*dev, host.data(), host.size() * sizeof(T), hipMemcpyHostToDevice), NUTS_E_DEVICE);
    return NUTS_OK;
}

template <typename T>
int build_device_data(nuts_target* t, const nuts_target_desc* desc)
{
    const int64_t d = desc->dim;
    switch (desc->kind) {
    case NUTS_TARGET_STD_NORMAL:
        return NUTS_OK;
    case NUTS_TARGET_GAUSS_DENSE_PRECISION: {
        const T* P = static_cast<const T*>(desc->precision);
        std::vector<T> PT((size_t)d * d);
        for (int64_t i = 0; i < d; ++i)
            for (int64_t k = 0; k < d; ++k) PT[(size_t)k * d + i] = P[(size_t)i * d + k];
        // structure: a matrix that is exactly zero beyond kBandHalf off-diagonals is also kept as a band
        int64_t half = 0;
        for (int64_t i = 0; i < d; ++i)
            for (int64_t k = 0; k < d; ++k)
                if (P[(size_t)i * d + k] != (T)0 && std::llabs(i - k) > half) half = std::llabs(i - k);
        if (half <= nuts::kBandHalf && d <= nuts::kBandRows) {
            const int w = 2 * nuts::kBandHalf + 1;
            std::vector<T> band((size_t)nuts::kBandRows * w, (T)0);
            for (int64_t i = 0; i < d; ++i)
                for (int64_t k = std::max<int64_t>(0, i - nuts::kBandHalf); k <= std::min<int64_t>(d - 1, i + nuts::kBandHalf); ++k)
                    band[(size_t)i * w + (size_t)(k - i + nuts::kBandHalf)] = P[(size_t)i * d + k];
            int rc = upload(band, &t->dBand);
            if (rc) return rc;
        }
        if (d <= nuts::kDenseMaxDim) {
            std::vector<double> ftab;
            nuts::build_softplus_table(&ftab);
            int rc = upload(ftab, &t->dFtab);
            if (rc) return rc;
        }
        if (sizeof(T) == sizeof(double) && d <= nuts::kQuadMaxDim) {
            std::vector<double> op;
            nuts::quad_pack_operands(reinterpret_cast<const double*>(P), d, &t->quad, &op);
            void* dev = nullptr;
            int rc = upload(op, &dev);
            if (rc) return rc;
            t->quad.ops = static_cast<double*>(dev);
        }
        return upload(PT, &t->dPT);
    }
    case NUTS_TARGET_GAUSS_DIAG: {
        const T* s = static_cast<const T*>(desc->scales);
        std::vector<T> w((size_t)d);
        for (int64_t i = 0; i < d; ++i) w[(size_t)i] = (T)(1.0 / ((double)s[i] * (double)s[i]));
        return upload(w, &t->dInvVar);
    }
    case NUTS_TARGET_LOGISTIC_REGRESSION: {
        const T* X = static_cast<const T*>(desc->X);
        const T* y = static_cast<const T*>(desc->y);
        const int64_t n = desc->n_data;
        std::vector<T> Xh(X, X + (size_t)n * d), yh(y, y + n), XT((size_t)n * d);
        for (int64_t r = 0; r < n; ++r)
            for (int64_t k = 0; k < d; ++k) XT[(size_t)k * n + r] = X[(size_t)r * d + k];
        int rc = upload(Xh, &t->dX);
        if (rc) return rc;
        rc = upload(XT, &t->dXT);
        if (rc) return rc;
        rc = upload(yh, &t->dY);
        if (rc) return rc;
        if (sizeof(T) == sizeof(double) && nuts::tile_supports_shape(d, n)) {
            std::vector<double> op, colsum, ftab;
            nuts::tile_pack_operands(reinterpret_cast<const double*>(X), reinterpret_cast<const double*>(y), n, d,
                                     &t->tile, &op, &colsum);
            nuts::build_softplus_table(&ftab);
            {
                std::vector<double> logtab;
                nuts::build_log_table(&logtab);
                ftab.insert(ftab.end(), logtab.begin(), logtab.end());
            }
            void* dev = nullptr;
            rc = upload(op, &dev);
            if (rc) return rc;
            t->tile.base = static_cast<double*>(dev);
            rc = upload(colsum, &dev);
            if (rc) return rc;
            t->tile.colsum = static_cast<double*>(dev);
            rc = upload(ftab, &dev);
            if (rc) return rc;
            t->tile.ftab = static_cast<double*>(dev);
        }
        if (sizeof(T) == sizeof(float) && nuts::grid_supports_shape(d)) {
            std::vector<float> op;
            nuts::grid_pack_operands(reinterpret_cast<const float*>(X), reinterpret_cast<const float*>(y), n, d, &t->grid, &op);
            void* dev = nullptr;
            rc = upload(op, &dev);
            if (rc) return rc;
            t->grid.ops = static_cast<float*>(dev);
        }
        return NUTS_OK;
    }
    default:
        return fail(NUTS_E_INVALID_ARG, "unknown target kind %d", desc->kind);
    }
}

template <typename T>
int check_values(const nuts_target_desc* desc)
{
    const int64_t d = desc->dim;
    if (desc->kind == NUTS_TARGET_GAUSS_DENSE_PRECISION) {
        const T* P = static_cast<const T*>(desc->precision);
        for (int64_t i = 0; i < d * d; ++i)
            if (!std::isfinite((double)P[i])) return fail(NUTS_E_INVALID_ARG, "precision[%lld] is not finite", (long long)i);
    } else if (desc->kind == NUTS_TARGET_GAUSS_DIAG) {
        const T* s = static_cast<const T*>(desc->scales);
        for (int64_t i = 0; i < d; ++i)
            if (!(s[i] > 0) || !std::isfinite((double)s[i]))
                return fail(NUTS_E_INVALID_ARG, "scales[%lld] must be finite and > 0", (long long)i);
    } else if (desc->kind == NUTS_TARGET_LOGISTIC_REGRESSION) {
        const T* X = static_cast<const T*>(desc->X);
        const T* y = static_cast<const T*>(desc->y);
        for (int64_t i = 0; i < desc->n_data * d; ++i)
            if (!std::isfinite((double)X[i])) return fail(NUTS_E_INVALID_ARG, "X[%lld] is not finite", (long long)i);
        for (int64_t i = 0; i < desc->n_data; ++i)
            if (!(y[i] == (T)0 || y[i] == (T)1)) return fail(NUTS_E_INVALID_ARG, "y[%lld] is not 0 or 1", (long long)i);
    }
    return NUTS_OK;
}

void release(nuts_target* t)
{
    if (!t) return;
    if (t->device >= 0) {
        (void)hipFree(t->dPT);
        (void)hipFree(t->dBand);
        (void)hipFree(t->dFtab);
        (void)hipFree(t->dInvVar);
        (void)hipFree(t->dX);
        (void)hipFree(t->dXT);
        (void)hipFree(t->dY);
        (void)hipFree(t->tile.base);
        (void)hipFree(t->grid.ops);
        (void)hipFree(t->quad.ops);
        (void)hipFree(t->tile.ftab);
        (void)hipFree(t->tile.colsum);
        (void)hipFree(t->workspace);
        (void)hipFree(t->carry);
        (void)hipFree(t->counters);
        if (t->ev_start) (void)hipEventDestroy(t->ev_start);
        if (t->ev_stop) (void)hipEventDestroy(t->ev_stop);
        if (t->ev_fork) (void)hipEventDestroy(t->ev_fork);
        for (hipEvent_t e : t->ev_join)
            if (e) (void)hipEventDestroy(e);
        for (hipStream_t q : t->side_stream)
            if (q) (void)hipStreamDestroy(q);
        for (hipEvent_t e : t->ev_batch)
            if (e) (void)hipEventDestroy(e);
        if (t->halted_host) (void)hipHostFree(t->halted_host);
    }
    delete t;
}

int ensure_device(nuts_target* t)
{
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || count < 1)
        return fail(NUTS_E_DEVICE, "no HIP device available (this library has no CPU path)");
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev), NUTS_E_DEVICE);
    if (t->device >= 0 && t->device != dev)
        return fail(NUTS_E_INVALID_ARG, "target was created on device %d, current device is %d", t->device, dev);
    t->device = dev;
    int rc = resolve_scratch(dev);
    if (rc) return rc;
    if (!t->counters) HIP_TRY(hipMalloc((void**)&t->counters, nuts::kCtrCount * sizeof(unsigned long long)), NUTS_E_ALLOC);
    if (!t->ev_start) HIP_TRY(hipEventCreate(&t->ev_start), NUTS_E_DEVICE);
    if (!t->ev_stop) HIP_TRY(hipEventCreate(&t->ev_stop), NUTS_E_DEVICE);
    return NUTS_OK;
}

int ensure_workspace(nuts_target* t, size_t bytes)
{
    if (t->static_call) {  // no allocation: the workspace is the device's static array, or the call is refused
        if (bytes > (size_t)NUTS_STATIC_SCRATCH_BYTES - kStaticHeader)
            return fail(NUTS_E_UNSUPPORTED, "this run needs %zu bytes of scratch memory; nuts_sample_static has %zu",
                        bytes, (size_t)NUTS_STATIC_SCRATCH_BYTES - kStaticHeader);
        t->ws_cur = reinterpret_cast<char*>(g_scratch_ptr[t->device]) + kStaticHeader;
        return NUTS_OK;
    }
    t->ws_cur = t->workspace;
    if (bytes <= t->workspace_bytes) return NUTS_OK;
    if (t->workspace) {
        HIP_TRY(hipDeviceSynchronize(), NUTS_E_DEVICE);
        (void)hipFree(t->workspace);
        t->workspace = nullptr;
        t->workspace_bytes = 0;
    }
    HIP_TRY(hipMalloc((void**)&t->workspace, bytes), NUTS_E_ALLOC);
    t->workspace_bytes = bytes;
    t->ws_cur = t->workspace;
    return NUTS_OK;
}

// The logistic table of the weight merges (wave, element-wise, dense and grid kernels).  Built when the
// target is created if a device is there, else at the first regular launch; never by nuts_sample_static.
int ensure_ftab(nuts_target* t)
{
    if (t->dFtab) return NUTS_OK;
    if (t->static_call)
        return fail(NUTS_E_UNSUPPORTED, "the target was created without a GPU: nuts_sample_static cannot build its tables");
    std::vector<double> ftab;
    nuts::build_softplus_table(&ftab);
    return upload(ftab, &t->dFtab);
}

__global__ void zero_counters_kernel(unsigned long long* c)
{
    if (threadIdx.x < nuts::kCtrCount) c[threadIdx.x] = 0ull;
}

// After every launch: the wave and element-wise kernels hold `slots` chain slots for as long as the
// busiest of them works, so that many slots x its gradient count were issued; the chain queue restarts.
__global__ void close_launch_kernel(unsigned long long* c, unsigned long long slots)
{
    if (threadIdx.x == 0) {
        c[nuts::kCtrIssued] += slots * c[nuts::kCtrSlotMax];
        c[nuts::kCtrSlotMax] = 0ull;
        c[nuts::kCtrQueue] = 0ull;
    }
}

int next_pow2(int x)
{
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

template <typename T>
nuts::DevTarget<T> dev_target(const nuts_target* t)
{
    nuts::DevTarget<T> g{};
    g.kind = t->kind;
    g.d = (int)t->dim;
    g.dstride = (int)((t->dim + 15) / 16 * 16);
    g.kl = next_pow2((int)(t->dim < 64 ? t->dim : 64));
    g.n = (long)t->n;
    g.PT = static_cast<const T*>(t->dPT);
    g.band = static_cast<const T*>(t->dBand);
    g.inv_var = static_cast<const T*>(t->dInvVar);
    g.X = static_cast<const T*>(t->dX);
    g.XT = static_cast<const T*>(t->dXT);
    g.y = static_cast<const T*>(t->dY);
    g.prior_prec = 1.0 / (t->prior_scale * t->prior_scale);
    return g;
}

template <typename T>
int launch_wave(nuts_target* t, nuts::DevSample sa)
{
    nuts::DevTarget<T> tg = dev_target<T>(t);
    const int waves_per_block = 4, threads = waves_per_block * nuts::kWave;
    size_t lds_bytes = (size_t)waves_per_block * tg.dstride * sizeof(T);
    if (lds_bytes > 64 * 1024) return fail(NUTS_E_UNSUPPORTED, "dim %lld too large for the wave kernel", (long long)t->dim);
    const size_t mat_bytes = (size_t)t->dim * t->dim * sizeof(T);
    if (t->kind == NUTS_TARGET_GAUSS_DENSE_PRECISION && lds_bytes + mat_bytes <= 128 * 1024) {
        tg.lds_matrix = 1;
        lds_bytes += mat_bytes;
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(nuts::nuts_wave_kernel<T>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes), NUTS_E_DEVICE);
    }
    size_t slot = ((size_t)nuts::wave_num_vectors(sa.max_depth) * tg.dstride * sizeof(T) + 15) & ~(size_t)15;
    if (t->kind == NUTS_TARGET_LOGISTIC_REGRESSION) slot += (size_t)t->n * sizeof(double);
    slot = (slot + 255) & ~(size_t)255;
    int per_cu = 0, cus = 0;
    HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, nuts::nuts_wave_kernel<T>, threads, lds_bytes),
            NUTS_E_DEVICE);
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, t->device), NUTS_E_DEVICE);
    if (per_cu < 1) per_cu = 1;
    long blocks = (sa.n_chains + waves_per_block - 1) / waves_per_block;
    const long resident = (long)per_cu * cus;
    if (blocks > resident) blocks = resident;
    int rc = ensure_workspace(t, slot * (size_t)blocks * waves_per_block);
    if (rc) return rc;
    sa.workspace = t->ws_cur;
    sa.slot_bytes = slot;
    hipLaunchKernelGGL(nuts::nuts_wave_kernel<T>, dim3((unsigned)blocks), dim3(threads), lds_bytes, g_stream, tg, sa);
    HIP_TRY(hipGetLastError(), NUTS_E_DEVICE);
    t->last_variant = NUTS_VARIANT_WAVE;
    t->last_grid = (int)blocks;
    t->last_slots = blocks * waves_per_block < sa.n_chains ? blocks * waves_per_block : sa.n_chains;  // waves that get a chain
    return NUTS_OK;
}

// Largest dimension the register-resident element-wise kernel takes, per dtype.
int elem_max_dim(int dtype) { return dtype == NUTS_F64 ? 512 : 1024; }

bool elem_eligible(const nuts_target* t)
{
    return (t->kind == NUTS_TARGET_STD_NORMAL || t->kind == NUTS_TARGET_GAUSS_DIAG) && t->dim <= elem_max_dim(t->dtype);
}

template <typename T, int kVpl>
int launch_elem_inst(nuts_target* t, nuts::DevSample sa)
{
    nuts::DevTarget<T> tg = dev_target<T>(t);
    const int waves_per_block = 4, threads = waves_per_block * nuts::kWave;
    size_t slot = (size_t)nuts::elem_num_vectors(sa.max_depth) * tg.dstride * sizeof(T);
    slot = (slot + 255) & ~(size_t)255;
    int per_cu = 0, cus = 0;
    HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, nuts::nuts_elem_kernel<T, kVpl>, threads, 0), NUTS_E_DEVICE);
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, t->device), NUTS_E_DEVICE);
    if (per_cu < 1) per_cu = 1;
    long blocks = (sa.n_chains + waves_per_block - 1) / waves_per_block;
    const long resident = (long)per_cu * cus;
    if (blocks > resident) blocks = resident;
    int rc = ensure_workspace(t, slot * (size_t)blocks * waves_per_block);
    if (rc) return rc;
    sa.workspace = t->ws_cur;
    sa.slot_bytes = slot;
    rc = ensure_ftab(t);
    if (rc) return rc;
    hipLaunchKernelGGL((nuts::nuts_elem_kernel<T, kVpl>), dim3((unsigned)blocks), dim3(threads), 0, g_stream, tg, sa,
                       static_cast<const double*>(t->dFtab));
    HIP_TRY(hipGetLastError(), NUTS_E_DEVICE);
    t->last_variant = NUTS_VARIANT_ELEM;
    t->last_grid = (int)blocks;
    t->last_slots = blocks * waves_per_block < sa.n_chains ? blocks * waves_per_block : sa.n_chains;  // waves that get a chain
    return NUTS_OK;
}

int launch_elem(nuts_target* t, const nuts::DevSample& sa)
{
    if (t->dtype == NUTS_F64) return t->dim <= 128 ? launch_elem_inst<double, 2>(t, sa) : launch_elem_inst<double, 8>(t, sa);
    return t->dim <= 256 ? launch_elem_inst<float, 4>(t, sa) : launch_elem_inst<float, 16>(t, sa);
}

bool dense_eligible(const nuts_target* t)
{
    return t->kind == NUTS_TARGET_GAUSS_DENSE_PRECISION && t->dim <= nuts::kDenseMaxDim;
}

template <typename T, bool kBanded>
int launch_dense_inst(nuts_target* t, nuts::DevSample sa)
{
    using namespace nuts;
    DevTarget<T> tg = dev_target<T>(t);
    const int threads = kDenseWaves * kWave;
    size_t lds_bytes = ((size_t)(kBanded ? 0 : t->dim) * kDensePitch +
                        (size_t)kDenseWaves * (kDensePitch + 2 * kBandHalf)) * sizeof(T);
    lds_bytes = (lds_bytes + 15) & ~(size_t)15;
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void*>(nuts_dense_kernel<T, kBanded>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes), NUTS_E_DEVICE);
    size_t slot = (size_t)dense_num_vectors(sa.max_depth) * kDensePitch * sizeof(T);
    slot = (slot + 255) & ~(size_t)255;
    int per_cu = 0, cus = 0;
    HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, (nuts_dense_kernel<T, kBanded>), threads, lds_bytes), NUTS_E_DEVICE);
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, t->device), NUTS_E_DEVICE);
    if (per_cu < 1) per_cu = 1;
    long blocks = (sa.n_chains + kDenseWaves - 1) / kDenseWaves;
    const long resident = (long)per_cu * cus;
    if (blocks > resident) blocks = resident;
    int rc = ensure_workspace(t, slot * (size_t)blocks * kDenseWaves);
    if (rc) return rc;
    sa.workspace = t->ws_cur;
    sa.slot_bytes = slot;
    hipLaunchKernelGGL((nuts_dense_kernel<T, kBanded>), dim3((unsigned)blocks), dim3(threads), lds_bytes, g_stream, tg, sa);
    HIP_TRY(hipGetLastError(), NUTS_E_DEVICE);
    t->last_variant = NUTS_VARIANT_DENSE;
    t->last_grid = (int)blocks;
    t->last_slots = blocks * kDenseWaves < sa.n_chains ? blocks * kDenseWaves : sa.n_chains;
    return NUTS_OK;
}

template <typename T>
int launch_dense(nuts_target* t, const nuts::DevSample& sa)
{
    return t->dBand ? launch_dense_inst<T, true>(t, sa) : launch_dense_inst<T, false>(t, sa);
}

bool quad_eligible(const nuts_target* t, int max_depth)
{
    return t->kind == NUTS_TARGET_GAUSS_DENSE_PRECISION && t->dtype == NUTS_F64 && t->quad.ops != nullptr &&
           max_depth <= nuts::kQuadMaxDepth;
}

// Four chains per wavefront, four wavefronts per workgroup, one workgroup per compute unit (the matrix fills its LDS).
int launch_quad(nuts_target* t, nuts::DevSample sa)
{
    using namespace nuts;
    QuadArgs qa{t->quad.ops, t->quad.d, t->quad.n_r, t->quad.n_kb};
    size_t lds_bytes = quad_matrix_bytes(t->quad) + quad_stage_bytes();
    int cus = 0;
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, t->device), NUTS_E_DEVICE);
    const int per_block = kQuadWaves * kQuadChains;
    long blocks = (sa.n_chains + per_block - 1) / per_block;
    if (blocks > cus) blocks = cus;  // further chains wait in the queue
    // spread few chains over the compute units first: a wave with one chain still runs whole matrix instructions
    size_t slot = (size_t)quad_num_vectors(sa.max_depth) * kQuadVecLen * sizeof(double);
    int rc = ensure_workspace(t, slot * (size_t)blocks * per_block);
    if (rc) return rc;
    sa.workspace = t->ws_cur;
    sa.slot_bytes = slot;
    HIP_TRY(quad_launch(qa, sa, (int)blocks, lds_bytes, g_stream), NUTS_E_DEVICE);
    t->last_variant = NUTS_VARIANT_QUAD;
    t->last_grid = (int)blocks;
    t->last_slots = 0;
    return NUTS_OK;
}

bool grid_eligible(const nuts_target* t)
{
    return t->kind == NUTS_TARGET_LOGISTIC_REGRESSION && t->dtype == NUTS_F32 && t->grid.ops != nullptr;
}

// Rounds of (control, gradient) launches, enqueued in batches; the host waits for each batch
// and stops when every chain has halted, so this variant returns only when sampling is complete.
// Slots beyond the first 128 form further sets whose rounds run on streams that the target owns.
int launch_grid(nuts_target* t, nuts::DevSample sa)
{
    using namespace nuts;
    typedef WaveChain<float> Chain;
    DevTarget<float> tg = dev_target<float>(t);
    // at most 1024 chains are resident; a slot whose chain has finished takes the next one from the queue
    const int n_slots = sa.n_chains >= kGridMaxChains ? kGridMaxChains : (int)((sa.n_chains + 3) / 4 * 4);
    const int n_sets = (n_slots + kGridSetChains - 1) / kGridSetChains;
    // consecutive sets share a stream: one control launch serves them all, one gradient launch each
    const int sets_per_stream = (n_sets + kGridMaxStreams - 1) / kGridMaxStreams;
    const int n_streams = (n_sets + sets_per_stream - 1) / sets_per_stream;
    int cus = 0;
    HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, t->device), NUTS_E_DEVICE);
    GridArgs ga{};
    ga.ops = t->grid.ops;
    ga.d = t->grid.d;
    ga.ks1 = t->grid.ks1;
    ga.mt = t->grid.mt;
    ga.tail = t->grid.tail;
    ga.n_tiles = t->grid.n_tiles;
    ga.n_rows = t->grid.n_rows;
    // a slice per compute unit, but at least two row tiles per slice unless the data are tiny: a launch's
    // fixed costs - operands of Theta, first tile, partial results - weigh more than its width (+13 % at
    // 10 000 rows and 1024 chains).  The split depends on the target only, never on the number of chains:
    // a chain's results must not change with the size of the batch it runs in.
    const int min_tiles = ga.n_tiles >= 64 ? 2 : 1;
    ga.n_slices = (ga.n_tiles + min_tiles - 1) / min_tiles;
    if (ga.n_slices > cus) ga.n_slices = cus;
    if (ga.n_slices > kGridMaxSlices) ga.n_slices = kGridMaxSlices;
    ga.counters = sa.counters;
    ga.chain_stride = n_sets * kGridSetChains;
    {
        int rc = ensure_ftab(t);
        if (rc) return rc;
    }
    ga.ftab = static_cast<const double*>(t->dFtab);

    // carve the workspace
    size_t off = 0;
    auto take = [&](size_t bytes) { const size_t o = off; off = (off + bytes + 255) & ~(size_t)255; return o; };
    const size_t chain_ws = ((size_t)wave_num_vectors(sa.max_depth) * tg.dstride * sizeof(float) + 255) & ~(size_t)255;
    const size_t o_theta = take((size_t)kGridFeatPad * ga.chain_stride * sizeof(float));
    const size_t o_gpart = take((size_t)ga.n_slices * ga.chain_stride * kGridFeatPad * sizeof(float));
    const size_t o_llpart = take((size_t)ga.n_slices * ga.chain_stride * sizeof(double));
    const size_t o_active = take((size_t)kGridMaxSets * kGridBatch * sizeof(int));
    const size_t o_halted = take((size_t)ga.chain_stride * sizeof(int));
    const size_t o_saved = take((size_t)ga.chain_stride * sizeof(Chain::Saved));
    const size_t o_chain = take(chain_ws * ga.chain_stride);
    int rc = ensure_workspace(t, off);
    if (rc) return rc;
    char* w = t->ws_cur;
    ga.b.theta_t = reinterpret_cast<float*>(w + o_theta);
    ga.b.g_part = reinterpret_cast<float*>(w + o_gpart);
    ga.b.ll_part = reinterpret_cast<double*>(w + o_llpart);
    ga.b.active_all = reinterpret_cast<int*>(w + o_active);
    ga.b.halted = reinterpret_cast<int*>(w + o_halted);
    ga.b.saved = w + o_saved;
    ga.b.chain_ws = w + o_chain;
    ga.b.chain_ws_bytes = chain_ws;

    // consecutive sets share a stream and its launches: same buffers (they own disjoint chain slots), own flags
    GridArgs span[kGridMaxStreams];
    hipStream_t stream[kGridMaxStreams] = {g_stream};
    for (int q = 0; q < n_streams; ++q) {
        span[q] = ga;
        span[q].slot_base = q * sets_per_stream * kGridSetChains;
        const int left = n_slots - span[q].slot_base, full = sets_per_stream * kGridSetChains;
        span[q].n_span_slots = left < full ? left : full;
    }
    if (n_streams > 1 && !t->ev_fork) HIP_TRY(hipEventCreateWithFlags(&t->ev_fork, hipEventDisableTiming), NUTS_E_DEVICE);
    for (int q = 1; q < n_streams; ++q) {
        if (!t->side_stream[q - 1]) HIP_TRY(hipStreamCreateWithFlags(&t->side_stream[q - 1], hipStreamNonBlocking), NUTS_E_DEVICE);
        if (!t->ev_join[q - 1]) HIP_TRY(hipEventCreateWithFlags(&t->ev_join[q - 1], hipEventDisableTiming), NUTS_E_DEVICE);
        stream[q] = t->side_stream[q - 1];
    }

    hipLaunchKernelGGL(nuts_grid_fill_kernel, dim3(64), dim3(256), 0, g_stream, reinterpret_cast<int*>(ga.b.theta_t),
                       kGridFeatPad * ga.chain_stride, 0);
    hipLaunchKernelGGL(nuts_grid_fill_kernel, dim3(4), dim3(256), 0, g_stream, ga.b.halted, ga.chain_stride, 1);
    if (n_streams > 1) {  // the side streams start after everything enqueued so far
        HIP_TRY(hipEventRecord(t->ev_fork, g_stream), NUTS_E_DEVICE);
        for (int q = 1; q < n_streams; ++q) HIP_TRY(hipStreamWaitEvent(stream[q], t->ev_fork, 0), NUTS_E_DEVICE);
    }
    // (a guard against a run that never ends: every chain one after the other, every tree full)
    const unsigned long long max_rounds =
        (unsigned long long)sa.n_chains * (unsigned long long)(sa.iter_end - sa.iter_begin) *
            ((unsigned long long)sa.leaf_steps * (1ull << sa.max_depth) + 2) + 8;
    // Batches are enqueued one ahead of the host's look at the "halted" flags, so the GPU never waits for
    // the host; when the flags of batch k say that everybody has halted, batch k + 1 (already enqueued)
    // consists of launches that return at once.  Each set's flags are copied on its own stream: the
    // streams meet again only at the end.
    if (!t->halted_host) HIP_TRY(hipHostMalloc((void**)&t->halted_host, 2 * kGridMaxChains * sizeof(int)), NUTS_E_ALLOC);
    for (hipEvent_t& e : t->ev_batch)
        if (!e) HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming), NUTS_E_DEVICE);
    unsigned long long rounds = 0;
    int first = 1;
    auto enqueue_batch = [&](int b) -> int {
        for (int q = 0; q < n_streams; ++q)
            hipLaunchKernelGGL(nuts_grid_fill_kernel, dim3(1), dim3(64), 0, stream[q],
                               ga.b.active_all + q * sets_per_stream * kGridBatch, sets_per_stream * kGridBatch, 0);
        for (int i = 0; i < kGridBatch; ++i) {
            for (int q = 0; q < n_streams; ++q) {
                hipLaunchKernelGGL(nuts_grid_control_kernel, dim3((unsigned)span[q].n_span_slots), dim3(256), 0, stream[q], tg, sa,
                                   span[q], i, first);
                grid_launch_grad_any(span[q], i, stream[q]);
            }
            first = 0;
            rounds += 1;
        }
        HIP_TRY(hipGetLastError(), NUTS_E_DEVICE);
        for (int q = 0; q < n_streams; ++q) {
            const int base = span[q].slot_base;
            const int count = ga.chain_stride - base < sets_per_stream * kGridSetChains ? ga.chain_stride - base : sets_per_stream * kGridSetChains;
            HIP_TRY(hipMemcpyAsync(t->halted_host + b * kGridMaxChains + base, ga.b.halted + base, count * sizeof(int),
                                   hipMemcpyDeviceToHost, stream[q]),
                    NUTS_E_DEVICE);
        }
        for (int q = 0; q < n_streams; ++q) HIP_TRY(hipEventRecord(t->ev_batch[kGridMaxStreams * b + q], stream[q]), NUTS_E_DEVICE);
        return NUTS_OK;
    };
    auto all_halted = [&](int b) -> int {  // 1 / 0, or a negative error code
        for (int q = 0; q < n_streams; ++q) HIP_TRY(hipEventSynchronize(t->ev_batch[kGridMaxStreams * b + q]), NUTS_E_DEVICE);
        for (int i = 0; i < n_sets * kGridSetChains; ++i)
            if (!t->halted_host[b * kGridMaxChains + i]) return 0;
        return 1;
    };
    rc = enqueue_batch(0);
    if (rc) return rc;
    for (int b = 0;; b ^= 1) {
        rc = enqueue_batch(b ^ 1);
        if (rc) return rc;
        const int done = all_halted(b);
        if (done < 0) return done;
        if (done) break;
        if (rounds > max_rounds + 2 * kGridBatch)
            return fail(NUTS_E_DEVICE, "grid sampler did not finish within %llu rounds", max_rounds);
    }
    for (int q = 1; q < n_streams; ++q) {  // the caller's stream continues after the side streams' last batch
        HIP_TRY(hipEventRecord(t->ev_join[q - 1], stream[q]), NUTS_E_DEVICE);
        HIP_TRY(hipStreamWaitEvent(g_stream, t->ev_join[q - 1], 0), NUTS_E_DEVICE);
    }
    hipLaunchKernelGGL(nuts_grid_finish_kernel, dim3(1), dim3(256), 0, g_stream, ga, sa, n_slots);
    HIP_TRY(hipGetLastError(), NUTS_E_DEVICE);
    t->last_variant = NUTS_VARIANT_GRID;
    t->last_grid = ga.n_slices;
    t->last_slots = 0;
    return NUTS_OK;
}

int launch_tile(nuts_target* t, nuts::DevSample sa)
{
    nuts::TileLaunch tl;
    nuts::tile_plan(t->tile, sa.n_chains, sa.max_depth, &tl);
    int rc = ensure_workspace(t, tl.workspace_bytes);
    if (rc) return rc;
    sa.workspace = t->ws_cur;
    sa.slot_bytes = tl.block_bytes;
    nuts::tile_launch(t->tile, sa, 1.0 / (t->prior_scale * t->prior_scale), tl, g_stream);
    HIP_TRY(hipGetLastError(), NUTS_E_DEVICE);
    t->last_variant = NUTS_VARIANT_TILE;
    t->last_grid = tl.blocks;
    t->last_slots = 0;
    return NUTS_OK;
}

bool tile_eligible(const nuts_target* t, int max_depth)
{
    return t->kind == NUTS_TARGET_LOGISTIC_REGRESSION && t->dtype == NUTS_F64 && t->tile.base != nullptr &&
           max_depth <= nuts::kTileMaxDepth;
}

}  // namespace

extern "C" {

const char* nuts_last_error(void) { return g_err; }

int nuts_tile_pack(const double* X, const double* y, int64_t n, int64_t d, nuts_tile_layout* layout, double* operands,
                   int64_t capacity)
{
    if (!X || !y || !layout) return fail(NUTS_E_INVALID_ARG, "nuts_tile_pack: null argument");
    if (!nuts::tile_supports_shape(d, n)) return fail(NUTS_E_INVALID_ARG, "nuts_tile_pack: shape outside the tile variant's range");
    nuts::TileData td;
    std::vector<double> op, colsum;
    nuts::tile_pack_operands(X, y, n, d, &td, &op, &colsum);
    layout->ks1 = td.ks1;
    layout->mt = td.mt;
    layout->n_tiles = td.n_tiles;
    layout->n_alloc_tiles = td.n_alloc_tiles;
    layout->const_col = td.z0_col;
    layout->reserved = 0;
    layout->const_val = td.z0_val;
    layout->n_pad = td.n_pad;
    layout->operand_doubles = (int64_t)op.size();
    if (operands) {
        if (capacity < (int64_t)op.size()) return fail(NUTS_E_INVALID_ARG, "nuts_tile_pack: operands buffer too small");
        std::memcpy(operands, op.data(), op.size() * sizeof(double));
    }
    return NUTS_OK;
}

int nuts_set_stream(void* hip_stream)
{
    g_stream = static_cast<hipStream_t>(hip_stream);
    return NUTS_OK;
}

int nuts_create_target(const nuts_target_desc* desc, nuts_target** out)
{
    if (!desc || !out) return fail(NUTS_E_INVALID_ARG, "desc and out must not be NULL");
    if (desc->dtype != NUTS_F32 && desc->dtype != NUTS_F64) return fail(NUTS_E_INVALID_ARG, "unknown dtype %d", desc->dtype);
    if (desc->kind < NUTS_TARGET_STD_NORMAL || desc->kind > NUTS_TARGET_LOGISTIC_REGRESSION)
        return fail(NUTS_E_INVALID_ARG, "unknown target kind %d", desc->kind);
    if (desc->dim < 1 || desc->dim > (1 << 24)) return fail(NUTS_E_INVALID_ARG, "dim must be in [1, 2^24]");
    if (desc->kind == NUTS_TARGET_GAUSS_DENSE_PRECISION && !desc->precision)
        return fail(NUTS_E_INVALID_ARG, "precision must not be NULL");
    if (desc->kind == NUTS_TARGET_GAUSS_DIAG && !desc->scales) return fail(NUTS_E_INVALID_ARG, "scales must not be NULL");
    if (desc->kind == NUTS_TARGET_LOGISTIC_REGRESSION) {
        if (!desc->X || !desc->y) return fail(NUTS_E_INVALID_ARG, "X and y must not be NULL");
        if (desc->n_data < 1 || desc->n_data > (1ll << 31) - 64) return fail(NUTS_E_INVALID_ARG, "n_data out of range");
        if (!(desc->prior_scale > 0.0) || !std::isfinite(desc->prior_scale))
            return fail(NUTS_E_INVALID_ARG, "prior_scale must be finite and > 0");
    }
    int rc = desc->dtype == NUTS_F64 ? check_values<double>(desc) : check_values<float>(desc);
    if (rc) return rc;

    nuts_target* t = new (std::nothrow) nuts_target();
    if (!t) return fail(NUTS_E_ALLOC, "out of host memory");
    t->kind = desc->kind;
    t->dtype = desc->dtype;
    t->dim = desc->dim;
    t->n = desc->kind == NUTS_TARGET_LOGISTIC_REGRESSION ? desc->n_data : 0;
    t->prior_scale = desc->kind == NUTS_TARGET_LOGISTIC_REGRESSION ? desc->prior_scale : 1.0;
    int n_dev = 0;
    const bool have_device = hipGetDeviceCount(&n_dev) == hipSuccess && n_dev >= 1;
    if (desc->kind != NUTS_TARGET_STD_NORMAL || have_device) {  // the standard normal has no data: it needs no device yet
        rc = ensure_device(t);
        if (!rc) rc = desc->dtype == NUTS_F64 ? build_device_data<double>(t, desc) : build_device_data<float>(t, desc);
        if (!rc) rc = ensure_ftab(t);
        if (rc) {
            release(t);
            return rc;
        }
    }
    *out = t;
    return NUTS_OK;
}

int nuts_destroy_target(nuts_target* t)
{
    release(t);
    return NUTS_OK;
}

}  // extern "C"

namespace {

// Body of nuts_sample_ex and nuts_sample_static.  With use_static the call takes its workspace and counters from
// the device's static scratch array and refuses whatever would need an allocation.
int sample_impl(const nuts_target* target, int64_t n_chains, int64_t n_iters, double step_size,
                int32_t max_tree_depth, uint64_t seed, const nuts_sample_options* options, void* out_states,
                int32_t* out_tree_depths, int32_t* out_n_leapfrog, bool use_static)
{
    if (!target) return fail(NUTS_E_INVALID_ARG, "target must not be NULL");
    if (n_chains < 1 || n_chains > (1ll << 31) - 1) return fail(NUTS_E_INVALID_ARG, "n_chains must be in [1, 2^31)");
    if (n_iters < 1 || n_iters > (1ll << 31) - 1) return fail(NUTS_E_INVALID_ARG, "n_iters must be in [1, 2^31)");
    if (!(step_size > 0.0) || !std::isfinite(step_size)) return fail(NUTS_E_INVALID_ARG, "step_size must be finite and > 0");
    if (max_tree_depth < 1 || max_tree_depth > 20) return fail(NUTS_E_INVALID_ARG, "max_tree_depth must be in [1, 20]");
    nuts_sample_options opt{};
    if (options) opt = *options;
    if (opt.first_chain < 0 || opt.first_chain + n_chains > (1ll << 32))
        return fail(NUTS_E_INVALID_ARG, "chain ids must fit in 32 bits");
    if (opt.variant < NUTS_VARIANT_AUTO || opt.variant > NUTS_VARIANT_QUAD)
        return fail(NUTS_E_INVALID_ARG, "unknown variant %d", opt.variant);
    if (opt.schedule != NUTS_SCHEDULE_FREE && opt.schedule != NUTS_SCHEDULE_TRAJECTORY)
        return fail(NUTS_E_INVALID_ARG, "unknown schedule %d", opt.schedule);
    if (opt.sampler != NUTS_SAMPLER_MULTINOMIAL && opt.sampler != NUTS_SAMPLER_SLICE)
        return fail(NUTS_E_INVALID_ARG, "unknown sampler %d", opt.sampler);
    if (opt.leaf_steps < 0 || opt.leaf_steps > NUTS_MAX_LEAF_STEPS)
        return fail(NUTS_E_INVALID_ARG, "leaf_steps must be in [1, %d] (0 = 1)", NUTS_MAX_LEAF_STEPS);
    const int leaf_steps = opt.leaf_steps == 0 ? 1 : opt.leaf_steps;
    nuts_target* t = const_cast<nuts_target*>(target);  // the scratch cache is logically mutable
    if (opt.variant == NUTS_VARIANT_TILE && !tile_eligible(t, max_tree_depth))
        return fail(NUTS_E_UNSUPPORTED,
                    "the tile kernel needs binary64 logistic regression with dim <= %d and max_tree_depth <= %d",
                    nuts::kTileMaxDim, nuts::kTileMaxDepth);

    if (opt.variant == NUTS_VARIANT_ELEM && !elem_eligible(t))
        return fail(NUTS_E_UNSUPPORTED, "the element-wise kernel needs a standard-normal or diagonal-Gaussian target with dim <= %d",
                    elem_max_dim(t->dtype));

    if (opt.variant == NUTS_VARIANT_GRID && !grid_eligible(t))
        return fail(NUTS_E_UNSUPPORTED, "the grid kernels need binary32 logistic regression with dim <= %d", nuts::kGridMaxDim);

    if (opt.variant == NUTS_VARIANT_QUAD && !quad_eligible(t, max_tree_depth))
        return fail(NUTS_E_UNSUPPORTED, "the quad kernel needs a binary64 dense Gaussian target with dim <= %d and max_tree_depth <= %d",
                    nuts::kQuadMaxDim, nuts::kQuadMaxDepth);

    if (opt.variant == NUTS_VARIANT_DENSE && !dense_eligible(t))
        return fail(NUTS_E_UNSUPPORTED, "the dense-Gaussian register kernel needs a dense Gaussian target with dim <= %d",
                    nuts::kDenseMaxDim);

    const bool use_tile = opt.variant == NUTS_VARIANT_TILE || (opt.variant == NUTS_VARIANT_AUTO && tile_eligible(t, max_tree_depth));
    const bool use_elem = opt.variant == NUTS_VARIANT_ELEM || (opt.variant == NUTS_VARIANT_AUTO && elem_eligible(t));
    // the grid kernels pay two launches per round; measured against the wave kernel they win from a few thousand
    // multiply-adds per gradient upwards (N d = 800: 2-5 times slower; 25 000: 3-7 times faster, at 8 to 1024 chains)
    const bool use_grid = opt.variant == NUTS_VARIANT_GRID ||
                          (opt.variant == NUTS_VARIANT_AUTO && grid_eligible(t) && t->n * t->dim >= (1 << 14));
    // A precision matrix that is not banded goes to the matrix cores, four chains per wavefront, once there are
    // enough chains to give every compute unit several (below that the one-chain-per-wavefront kernel spreads
    // them over more SIMDs; measured crossover, see the profile summary of the quad kernel)
    const bool use_quad = opt.variant == NUTS_VARIANT_QUAD ||
                          (opt.variant == NUTS_VARIANT_AUTO && quad_eligible(t, max_tree_depth) && !t->dBand &&
                           n_chains >= nuts::kQuadAutoChains);
    const bool use_dense = !use_quad && (opt.variant == NUTS_VARIANT_DENSE || (opt.variant == NUTS_VARIANT_AUTO && dense_eligible(t)));

    int rc = NUTS_OK;
    if (use_static) {
        // nothing below may allocate: the target must already hold its device data, counters and events
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess) return fail(NUTS_E_DEVICE, "no HIP device available (this library has no CPU path)");
        if (t->device < 0 || !t->counters || !t->ev_start || !t->ev_stop)
            return fail(NUTS_E_UNSUPPORTED, "the target was created without a GPU: nuts_sample_static cannot set it up");
        if (t->device != dev)
            return fail(NUTS_E_INVALID_ARG, "target was created on device %d, current device is %d", t->device, dev);
        if (!g_scratch_ptr[dev]) return fail(NUTS_E_DEVICE, "static scratch of device %d was not resolved", dev);
        if (use_grid && !use_dense && !use_tile)
            return fail(NUTS_E_UNSUPPORTED, "the grid kernels own streams and pinned host memory: not available without allocation");
        if (opt.schedule == NUTS_SCHEDULE_TRAJECTORY && !out_states)
            return fail(NUTS_E_UNSUPPORTED, "the trajectory schedule without out_states needs a carry buffer: pass out_states");
    } else {
        rc = ensure_device(t);
        if (rc) return rc;
    }
    t->static_call = use_static;
    t->counters_cur = use_static ? reinterpret_cast<unsigned long long*>(g_scratch_ptr[t->device]) : t->counters;

    nuts::DevSample sa{};
    sa.n_chains = (long)n_chains;
    sa.first_chain = (long)opt.first_chain;
    sa.n_iters = (int)n_iters;
    sa.max_depth = max_tree_depth;
    sa.leaf_steps = leaf_steps;
    sa.sampler = opt.sampler;
    sa.eps = step_size;
    sa.key0 = (uint32_t)(seed & 0xffffffffu);
    sa.key1 = (uint32_t)(seed >> 32);
    sa.out_states = out_states;
    sa.out_depths = out_tree_depths;
    sa.out_nleap = out_n_leapfrog;
    sa.init_states = opt.init_states;
    sa.counters = t->counters_cur;

    // the counters start at zero (a fill kernel, so that the call can sit inside a captured graph)
    hipLaunchKernelGGL(zero_counters_kernel, dim3(1), dim3(64), 0, g_stream, t->counters_cur);
    HIP_TRY(hipGetLastError(), NUTS_E_DEVICE);

    auto launch = [&](const nuts::DevSample& s) -> int {
        int r;
        if (use_quad)
            r = launch_quad(t, s);
        else if (use_dense)
            r = t->dtype == NUTS_F64 ? launch_dense<double>(t, s) : launch_dense<float>(t, s);
        else if (use_tile)
            r = launch_tile(t, s);
        else if (use_grid)
            r = launch_grid(t, s);
        else if (use_elem)
            r = launch_elem(t, s);
        else
            r = t->dtype == NUTS_F64 ? launch_wave<double>(t, s) : launch_wave<float>(t, s);
        if (r) return r;
        hipLaunchKernelGGL(close_launch_kernel, dim3(1), dim3(64), 0, g_stream, t->counters_cur, (unsigned long long)t->last_slots);
        HIP_TRY(hipGetLastError(), NUTS_E_DEVICE);
        return NUTS_OK;
    };
    if (opt.schedule == NUTS_SCHEDULE_TRAJECTORY) {
        // every chain finishes iteration i before any chain starts iteration i + 1: one launch per
        // iteration; a launch starts from the states the one before wrote.  A caller that wants no
        // states still needs them for that: they go to a one-iteration carry buffer instead.
        const size_t carry_bytes = (size_t)n_chains * (size_t)t->dim * (t->dtype == NUTS_F64 ? 8 : 4);
        if (!use_static && !out_states && carry_bytes > t->carry_bytes) {
            if (t->carry) {
                HIP_TRY(hipDeviceSynchronize(), NUTS_E_DEVICE);
                (void)hipFree(t->carry);
                t->carry = nullptr;
                t->carry_bytes = 0;
            }
            HIP_TRY(hipMalloc(&t->carry, carry_bytes), NUTS_E_ALLOC);
            t->carry_bytes = carry_bytes;
        }
    }
    HIP_TRY(hipEventRecord(t->ev_start, g_stream), NUTS_E_DEVICE);
    if (opt.schedule == NUTS_SCHEDULE_TRAJECTORY) {
        const size_t row_bytes = (size_t)n_chains * (size_t)t->dim * (t->dtype == NUTS_F64 ? 8 : 4);
        for (int64_t i = 0; i < n_iters && !rc; ++i) {
            sa.iter_begin = (int)i;
            sa.iter_end = (int)i + 1;
            if (out_states) {
                if (i > 0) sa.init_states = static_cast<char*>(out_states) + (size_t)(i - 1) * row_bytes;
            } else {
                // the kernels address states as base + (iteration * n_chains + chain) * dim: shift the base so
                // that this iteration's row is the carry buffer (each chain reads its row before it writes it)
                sa.out_states = reinterpret_cast<void*>(reinterpret_cast<uintptr_t>(t->carry) - (uintptr_t)i * row_bytes);
                if (i > 0) sa.init_states = t->carry;
            }
            rc = launch(sa);
        }
    } else {
        sa.iter_begin = 0;
        sa.iter_end = (int)n_iters;
        rc = launch(sa);
    }
    if (rc) return rc;
    HIP_TRY(hipEventRecord(t->ev_stop, g_stream), NUTS_E_DEVICE);
    t->has_run = true;
    return NUTS_OK;
}

}  // namespace

extern "C" {

int nuts_sample_ex(const nuts_target* target, int64_t n_chains, int64_t n_iters, double step_size,
                   int32_t max_tree_depth, uint64_t seed, const nuts_sample_options* options, void* out_states,
                   int32_t* out_tree_depths, int32_t* out_n_leapfrog)
{
    return sample_impl(target, n_chains, n_iters, step_size, max_tree_depth, seed, options, out_states, out_tree_depths,
                       out_n_leapfrog, false);
}

int nuts_sample_static(const nuts_target* target, int64_t n_chains, int64_t n_iters, double step_size,
                       int32_t max_tree_depth, uint64_t seed, const nuts_sample_options* options, void* out_states,
                       int32_t* out_tree_depths, int32_t* out_n_leapfrog)
{
    return sample_impl(target, n_chains, n_iters, step_size, max_tree_depth, seed, options, out_states, out_tree_depths,
                       out_n_leapfrog, true);
}

int nuts_sample(const nuts_target* target, int64_t n_chains, int64_t n_iters, double step_size, int32_t max_tree_depth,
                uint64_t seed, void* out_states, int32_t* out_tree_depths, int32_t* out_n_leapfrog)
{
    return nuts_sample_ex(target, n_chains, n_iters, step_size, max_tree_depth, seed, nullptr, out_states,
                          out_tree_depths, out_n_leapfrog);
}

int nuts_get_stats(const nuts_target* target, nuts_stats* out)
{
    if (!target || !out) return fail(NUTS_E_INVALID_ARG, "target and out must not be NULL");
    if (!target->has_run) return fail(NUTS_E_INVALID_ARG, "no sampling call has been made on this target");
    HIP_TRY(hipEventSynchronize(target->ev_stop), NUTS_E_DEVICE);
    unsigned long long c[nuts::kCtrCount];
    HIP_TRY(hipMemcpy(c, target->counters_cur, sizeof(c), hipMemcpyDeviceToHost), NUTS_E_DEVICE);
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, target->ev_start, target->ev_stop), NUTS_E_DEVICE);
    out->leaf_slots_issued = c[nuts::kCtrIssued];
    out->leaf_slots_useful = c[nuts::kCtrUseful];
    out->extra_grad_evals = c[nuts::kCtrExtra];
    out->rounds = c[nuts::kCtrRounds];
    out->kernel_ms = ms;
    out->phase_ticks[0] = c[nuts::kCtrCycControl];
    out->phase_ticks[1] = c[nuts::kCtrCycGrad];
    out->phase_ticks[2] = c[nuts::kCtrCycPost];
    out->variant = target->last_variant;
    out->grid_blocks = target->last_grid;
    return NUTS_OK;
}

}  // extern "C"
