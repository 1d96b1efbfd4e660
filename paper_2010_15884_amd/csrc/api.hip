// C-ABI layer of libsysconv: argument validation, projection dispatch, status
// reporting.  Every check runs before the first HIP call, so the error paths
// work on a host without a GPU.
#include "sysconv.h"

#include "launch.h"

#include <limits.h>
#include <stdint.h>

namespace {

thread_local int g_last_hip_error = 0;

int hip_status(hipError_t e)
{
    if (e == hipSuccess) return SYS_OK;
    g_last_hip_error = (int)e;
    return SYS_ERR_HIP;
}

bool ranges_overlap(const void* a, size_t a_bytes, const void* b, size_t b_bytes)
{
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + b_bytes && b0 < a0 + a_bytes;
}

bool known_projection(int p)
{
    return p >= SYS_PROJ_AUTO && p <= SYS_PROJ_MFMA;
}

bool misaligned(const void* p) { return ((uintptr_t)p & 3u) != 0; }

// The 2-D kernels and their launchers round widths up to whole strips (at most 1024
// columns) in int arithmetic; rows longer than this would overflow there.
bool too_wide(int w) { return w > INT_MAX - 2048; }

}  // namespace

extern "C" {

int sys_conv1d(const float* d_x, size_t n, const float* h_w, int k, float* d_y, int projection,
               hipStream_t stream)
{
    if (!d_x || !h_w || !d_y) return SYS_ERR_NULL;
    if (k < 1 || (size_t)k > n) return SYS_ERR_SIZE;
    if (!known_projection(projection) || k > SYS_MAX_K1D) return SYS_ERR_UNSUPPORTED;
    if (misaligned(d_x) || misaligned(d_y)) return SYS_ERR_UNSUPPORTED;
    if (n > ((size_t)1 << 40)) return SYS_ERR_UNSUPPORTED;
    const size_t m = n - (size_t)k + 1;
    if (ranges_overlap(d_x, n * sizeof(float), d_y, m * sizeof(float))) return SYS_ERR_ALIAS;

    switch (projection) {
    case SYS_PROJ_AUTO:
        // Long filters are bound by the VALUs, where BFS issues the fewest instructions
        // (n = 2^26: k = 34: 110 / 109 us FBS / BFS, k = 36: 113 / 108, k = 48: 146 / 120,
        // k = 64: 208 / 142; up to k = 28 FBS sits on the copy rate and BFS 5-10 % above it).
        // On signals of 2 GB and more BFS, whose register groups do not overlap, is the
        // faster one at every k (n = 2^29: 739 / 709 us at k = 16, 744 / 708 at k = 5;
        // n = 2^28: level).
        if ((k >= 36 || n >= ((size_t)1 << 29)) && sysconv::has_conv1d_bfs(k))
            return hip_status(sysconv::launch_conv1d_bfs(d_x, n, h_w, k, d_y, stream));
        return hip_status(sysconv::launch_conv1d_fbs(d_x, n, h_w, k, d_y, stream));
    case SYS_PROJ_FBS: return hip_status(sysconv::launch_conv1d_fbs(d_x, n, h_w, k, d_y, stream));
    case SYS_PROJ_SBM: return hip_status(sysconv::launch_conv1d_sbm(d_x, n, h_w, k, d_y, stream));
    case SYS_PROJ_BFS:
        if (!sysconv::has_conv1d_bfs(k)) return SYS_ERR_UNSUPPORTED;
        return hip_status(sysconv::launch_conv1d_bfs(d_x, n, h_w, k, d_y, stream));
    case SYS_PROJ_BSM: return hip_status(sysconv::launch_conv1d_bsm(d_x, n, h_w, k, d_y, stream));
    case SYS_PROJ_FSM: return hip_status(sysconv::launch_conv1d_fsm(d_x, n, h_w, k, d_y, stream));
    case SYS_PROJ_FFS: return hip_status(sysconv::launch_conv1d_ffs(d_x, n, h_w, k, d_y, stream));
    default: return SYS_ERR_UNSUPPORTED;
    }
}

int sys_conv1d_strided(const float* d_x, size_t n, const float* h_w, int k, int stride, float* d_y, int projection,
                       hipStream_t stream)
{
    if (stride == 1) return sys_conv1d(d_x, n, h_w, k, d_y, projection, stream);
    if (!d_x || !h_w || !d_y) return SYS_ERR_NULL;
    if (k < 1 || (size_t)k > n || stride < 1) return SYS_ERR_SIZE;
    if (!known_projection(projection) || k > SYS_MAX_K1D) return SYS_ERR_UNSUPPORTED;
    if (!sys_conv1d_strided_has(projection, k, stride)) return SYS_ERR_UNSUPPORTED;
    if (misaligned(d_x) || misaligned(d_y)) return SYS_ERR_UNSUPPORTED;
    if (n > ((size_t)1 << 40)) return SYS_ERR_UNSUPPORTED;
    const size_t m = (n - (size_t)k) / (size_t)stride + 1;
    if (ranges_overlap(d_x, n * sizeof(float), d_y, m * sizeof(float))) return SYS_ERR_ALIAS;
    return hip_status(sysconv::launch_conv1d_fbs_stride2(d_x, n, h_w, k, d_y, stream));
}

int sys_conv1d_strided_has(int projection, int k, int stride)
{
    if (stride == 1) return sys_conv1d_has(projection, k);
    if (k < 1 || k > SYS_MAX_K1D || stride != 2) return 0;
    return (projection == SYS_PROJ_AUTO || projection == SYS_PROJ_FBS) ? 1 : 0;
}

namespace {
int stt_status(const sys_stt_design_t* d, int k, sysconv::SttPlan* plan)
{
    if (!d) return SYS_ERR_NULL;
    if (k < 1 || k > SYS_MAX_K1D) return SYS_ERR_SIZE;
    switch (sysconv::plan_stt(d->alloc, d->sched, d->x_passed != 0, d->dep_x, d->w_passed != 0, d->dep_w, d->dep_z, k,
                              plan)) {
    case sysconv::kSttOk: return SYS_OK;
    case sysconv::kSttTooLarge: return SYS_ERR_UNSUPPORTED;
    default: return SYS_ERR_DESIGN;
    }
}
}  // namespace

int sys_stt_check(const sys_stt_design_t* design, int k)
{
    return stt_status(design, k, nullptr);
}

int sys_conv1d_stt(const float* d_x, size_t n, const float* h_w, int k, float* d_y, const sys_stt_design_t* design,
                   hipStream_t stream)
{
    if (!d_x || !h_w || !d_y || !design) return SYS_ERR_NULL;
    if (k < 1 || (size_t)k > n) return SYS_ERR_SIZE;
    if (k > SYS_MAX_K1D) return SYS_ERR_UNSUPPORTED;
    sysconv::SttPlan plan;
    const int st = stt_status(design, k, &plan);
    if (st != SYS_OK) return st;
    if (misaligned(d_x) || misaligned(d_y)) return SYS_ERR_UNSUPPORTED;
    if (n > ((size_t)1 << 40)) return SYS_ERR_UNSUPPORTED;
    const size_t m = n - (size_t)k + 1;
    if (ranges_overlap(d_x, n * sizeof(float), d_y, m * sizeof(float))) return SYS_ERR_ALIAS;
    return hip_status(sysconv::launch_conv1d_stt(d_x, n, h_w, k, d_y, plan, stream));
}

int sys_conv1d_has(int projection, int k)
{
    if (k < 1 || k > SYS_MAX_K1D) return 0;
    switch (projection) {
    case SYS_PROJ_AUTO:
    case SYS_PROJ_FBS:
    case SYS_PROJ_SBM:
    case SYS_PROJ_BSM:
    case SYS_PROJ_FSM:
    case SYS_PROJ_FFS: return 1;
    case SYS_PROJ_BFS: return sysconv::has_conv1d_bfs(k) ? 1 : 0;
    default: return 0;                                                 // MFMA is 2-D only
    }
}

int sys_conv2d_has(int projection, int kh, int kw)
{
    if (kh < 1 || kw < 1 || kh > SYS_MAX_K2D || kw > SYS_MAX_K2D) return 0;
    switch (projection) {
    case SYS_PROJ_AUTO:
    case SYS_PROJ_FBS: return 1;
    case SYS_PROJ_BFS: return sysconv::has_conv2d_bfs(kh, kw) ? 1 : 0;
    case SYS_PROJ_SBM: return sysconv::has_conv2d_sbm(kh, kw) ? 1 : 0;
    case SYS_PROJ_MFMA: return sysconv::has_conv2d_mfma(kh, kw) ? 1 : 0;
    default: return 0;
    }
}

int sys_conv2d(const float* d_x, int h, int w, size_t x_pitch, const float* h_f, int kh, int kw, float* d_y,
               size_t y_pitch, int projection, hipStream_t stream)
{
    if (!d_x || !h_f || !d_y) return SYS_ERR_NULL;
    if (h < 1 || w < 1 || kh < 1 || kw < 1 || kh > h || kw > w) return SYS_ERR_SIZE;
    const int oh = h - kh + 1, ow = w - kw + 1;
    if (x_pitch < (size_t)w || y_pitch < (size_t)ow) return SYS_ERR_SIZE;
    if (!known_projection(projection) || kh > SYS_MAX_K2D || kw > SYS_MAX_K2D) return SYS_ERR_UNSUPPORTED;
    if (misaligned(d_x) || misaligned(d_y)) return SYS_ERR_UNSUPPORTED;
    if (too_wide(w) || x_pitch > ((size_t)1 << 31) || y_pitch > ((size_t)1 << 31)) return SYS_ERR_UNSUPPORTED;
    if (projection == SYS_PROJ_MFMA
        && (!sysconv::has_conv2d_mfma(kh, kw) || !sysconv::conv2d_mfma_taps_in_range(h_f, kh * kw)))
        return SYS_ERR_UNSUPPORTED;
    const size_t x_bytes = ((size_t)(h - 1) * x_pitch + (size_t)w) * sizeof(float);
    const size_t y_bytes = ((size_t)(oh - 1) * y_pitch + (size_t)ow) * sizeof(float);
    if (ranges_overlap(d_x, x_bytes, d_y, y_bytes)) return SYS_ERR_ALIAS;

    int proj = projection;
    // Measured on MI355X, square images of 1000 .. 10240 columns (us, 5x5: BFS / SBM / FBS): 2996^2 15.8 / 14.3 / 14.3,
    // 4092^2 25.9 / 28.7 / 27.1, 4604^2 33.9 / 36.4 / 32.5, 5996^2 57.2 / 57.0 / 51.1, 7164^2 81.0 / 83.6 / 75.1,
    // 8188^2 103 / 104 / 95.5, 10236^2 166 / 170 / 155.  Up to 6x6 the FBS tile kernels win by 3 - 17 % except where
    // the input pitch is a power of two of at most 16 KB (1024, 2048, 4096 columns): there single-strip order and the
    // BFS block kernel's 1 KB-aligned strips win by 4 - 12 %.  7x7: SBM by 2 - 12 %.  8x8 .. 11x11: SBM.  The rest: FBS.
    if (proj == SYS_PROJ_AUTO) {
        const size_t pitch_bytes = x_pitch * sizeof(float);
        const bool short_pow2_pitch = (pitch_bytes & (pitch_bytes - 1)) == 0 && pitch_bytes <= 16384;
        if (kh == kw && kh >= 2 && kh <= 6) proj = short_pow2_pitch ? SYS_PROJ_BFS : SYS_PROJ_FBS;
        else if (sysconv::has_conv2d_sbm(kh, kw) && kh >= 7) proj = SYS_PROJ_SBM;
        else proj = SYS_PROJ_FBS;
    }
    switch (proj) {
    case SYS_PROJ_FBS:
        return hip_status(sysconv::launch_conv2d_fbs(d_x, h, w, x_pitch, h_f, kh, kw, d_y, y_pitch, stream));
    case SYS_PROJ_BFS:
        if (!sysconv::has_conv2d_bfs(kh, kw)) return SYS_ERR_UNSUPPORTED;
        return hip_status(sysconv::launch_conv2d_bfs(d_x, h, w, x_pitch, h_f, kh, kw, d_y, y_pitch, stream));
    case SYS_PROJ_SBM:
        if (!sysconv::has_conv2d_sbm(kh, kw)) return SYS_ERR_UNSUPPORTED;
        return hip_status(sysconv::launch_conv2d_sbm(d_x, h, w, x_pitch, h_f, kh, kw, d_y, y_pitch, stream));
    case SYS_PROJ_MFMA:                                                // size and tap range were checked above
        return hip_status(sysconv::launch_conv2d_mfma(d_x, h, w, x_pitch, h_f, kh, kw, d_y, y_pitch, stream));
    default: return SYS_ERR_UNSUPPORTED;                               // BSM, FSM, FFS are 1-D only
    }
}

int sys_conv2d_strided(const float* d_x, int h, int w, size_t x_pitch, const float* h_f, int kh, int kw, int stride,
                       float* d_y, size_t y_pitch, int projection, hipStream_t stream)
{
    if (stride == 1) return sys_conv2d(d_x, h, w, x_pitch, h_f, kh, kw, d_y, y_pitch, projection, stream);
    if (!d_x || !h_f || !d_y) return SYS_ERR_NULL;
    if (h < 1 || w < 1 || kh < 1 || kw < 1 || kh > h || kw > w || stride < 1) return SYS_ERR_SIZE;
    const int oh = (h - kh) / stride + 1, ow = (w - kw) / stride + 1;
    if (x_pitch < (size_t)w || y_pitch < (size_t)ow) return SYS_ERR_SIZE;
    if (!known_projection(projection) || kh > SYS_MAX_K2D || kw > SYS_MAX_K2D) return SYS_ERR_UNSUPPORTED;
    if (!sys_conv2d_strided_has(projection, kh, kw, stride)) return SYS_ERR_UNSUPPORTED;
    if (misaligned(d_x) || misaligned(d_y)) return SYS_ERR_UNSUPPORTED;
    if (too_wide(w) || x_pitch > ((size_t)1 << 31) || y_pitch > ((size_t)1 << 31)) return SYS_ERR_UNSUPPORTED;
    const size_t x_bytes = ((size_t)(h - 1) * x_pitch + (size_t)w) * sizeof(float);
    const size_t y_bytes = ((size_t)(oh - 1) * y_pitch + (size_t)ow) * sizeof(float);
    if (ranges_overlap(d_x, x_bytes, d_y, y_bytes)) return SYS_ERR_ALIAS;
    return hip_status(sysconv::launch_conv2d_fbs_stride2(d_x, h, w, x_pitch, h_f, kh, kw, d_y, y_pitch, stream));
}

int sys_conv2d_strided_has(int projection, int kh, int kw, int stride)
{
    if (stride == 1) return sys_conv2d_has(projection, kh, kw);
    if (kh < 1 || kw < 1 || kh > SYS_MAX_K2D || kw > SYS_MAX_K2D || stride != 2) return 0;
    return (projection == SYS_PROJ_AUTO || projection == SYS_PROJ_FBS) ? 1 : 0;
}

int sys_copy_f32(const float* d_src, float* d_dst, size_t n, hipStream_t stream)
{
    if (!d_src || !d_dst) return SYS_ERR_NULL;
    if (n < 1) return SYS_ERR_SIZE;
    if (misaligned(d_src) || misaligned(d_dst)) return SYS_ERR_UNSUPPORTED;
    if (ranges_overlap(d_src, n * sizeof(float), d_dst, n * sizeof(float))) return SYS_ERR_ALIAS;
    return hip_status(sysconv::launch_copy_f32(d_src, d_dst, n, stream));
}

long long sys_alu_yardstick_f32(float* d_out, int workgroups, int trips, hipStream_t stream)
{
    if (!d_out) return -(long long)SYS_ERR_NULL;
    if (workgroups < 1 || trips < 1 || workgroups > (1 << 20) || trips > (1 << 20)) return -(long long)SYS_ERR_SIZE;
    if (misaligned(d_out)) return -(long long)SYS_ERR_UNSUPPORTED;
    const int st = hip_status(sysconv::launch_alu_yardstick(d_out, workgroups, trips, stream));
    return st == SYS_OK ? sysconv::alu_yardstick_fmas(workgroups, trips) : -(long long)st;
}

const char* sys_status_string(int status)
{
    switch (status) {
    case SYS_OK: return "ok";
    case SYS_ERR_NULL: return "null pointer argument";
    case SYS_ERR_SIZE: return "invalid size (need 1 <= taps <= extent, pitch >= width)";
    case SYS_ERR_ALIAS: return "input and output ranges overlap";
    case SYS_ERR_UNSUPPORTED: return "unsupported size, alignment or projection";
    case SYS_ERR_HIP: return "HIP runtime error (see sys_last_hip_error)";
    case SYS_ERR_DESIGN: return "not a valid systolic design (dependence, singular transform or causality)";
    default: return "unknown status";
    }
}

const char* sys_projection_name(int projection)
{
    switch (projection) {
    case SYS_PROJ_AUTO: return "AUTO";
    case SYS_PROJ_FBS: return "FBS";
    case SYS_PROJ_BFS: return "BFS";
    case SYS_PROJ_SBM: return "SBM";
    case SYS_PROJ_BSM: return "BSM";
    case SYS_PROJ_FSM: return "FSM";
    case SYS_PROJ_FFS: return "FFS";
    case SYS_PROJ_MFMA: return "MFMA";
    default: return "?";
    }
}

int sys_last_hip_error(void) { return g_last_hip_error; }

int sys_version(void) { return 200; }

}  // extern "C"
