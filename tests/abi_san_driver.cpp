// Host-side checks of libsysconv for a build with -fsanitize=address,undefined (host code only): every
// argument check of the C ABI and the space-time-transform planner (the validity conditions of the paper's
// Section 2.2 and the launch plan derived from a design), driven with designs and sizes from the edges of
// what they accept.  Nothing here reaches a HIP call: every request is either answered by a query function
// or refused by the validation that precedes the launch, so the program runs on a host without a GPU.
// The "device" pointers are made-up addresses that validation must never dereference.
#include <limits.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <vector>

#define SYSCONV_NO_HIP_HEADER
#include "sysconv.h"

static int failures = 0;
#define EXPECT(expr, want) do { const int got_ = (expr); if (got_ != (want)) { \
    fprintf(stderr, "line %d: %s = %d (%s), expected %d\n", __LINE__, #expr, got_, sys_status_string(got_), (int)(want)); \
    ++failures; } } while (0)

static sys_stt_design_t design(int p0, int p1, int s0, int s1, int xon, int ex0, int ex1, int won, int ew0, int ew1,
                               int ez0, int ez1)
{
    sys_stt_design_t d;
    memset(&d, 0, sizeof d);
    d.alloc[0] = p0; d.alloc[1] = p1; d.sched[0] = s0; d.sched[1] = s1;
    d.x_passed = xon; d.dep_x[0] = ex0; d.dep_x[1] = ex1;
    d.w_passed = won; d.dep_w[0] = ew0; d.dep_w[1] = ew1;
    d.dep_z[0] = ez0; d.dep_z[1] = ez1;
    return d;
}

int main()
{
    float* const X = (float*)0x10000000;
    float* const Y = (float*)0x40000000;
    std::vector<float> taps(256, 1.0f);                            // exactly as many as the largest filter reads

    // ---- the six designs of Table 2 and five others: valid for every tap count the planner accepts
    const sys_stt_design_t valid[] = {
        design(1, 1, 0, 1, 1, -1, 1, 0, 0, 0, 0, 1),               // SBM
        design(0, 1, 1, 1, 0, 0, 0, 1, 1, 0, 0, 1),                // BSM
        design(0, 1, 1, -1, 1, 1, -1, 1, 1, 0, 0, -1),             // FSM
        design(1, 0, 1, 1, 0, 0, 0, 1, 1, 0, 0, 1),                // BFS
        design(1, 0, 2, 1, 1, 1, -1, 1, 1, 0, 0, 1),               // FFS
        design(1, 0, 0, 1, 1, -1, 1, 0, 0, 0, 0, 1),               // FBS
        design(1, 0, 1, 1, 0, 0, 0, 0, 0, 0, 0, 1),                // everything loaded, sums stay
        design(1, 1, 1, 2, 1, -1, 1, 0, 0, 0, 0, 1),               // SBM at half speed
        design(-1, 0, 0, 1, 1, -1, 1, 0, 0, 0, 0, 1),              // FBS, PE index against c
        design(0, -1, 1, -1, 1, 1, -1, 1, 1, 0, 0, -1),            // FSM mirrored
        design(1, 0, 0, -1, 1, 1, -1, 0, 0, 0, 0, -1),             // FBS, taps descending
    };
    for (const sys_stt_design_t& d : valid)
        for (int k = 1; k <= SYS_MAX_K1D; ++k) {
            const int st = sys_stt_check(&d, k);
            if (st != SYS_OK && st != SYS_ERR_UNSUPPORTED) {       // long filters may not fit 64 lanes: unsupported, never invalid
                fprintf(stderr, "valid design refused as %s at k=%d\n", sys_status_string(st), k);
                ++failures;
            }
        }
    EXPECT(sys_stt_check(&valid[0], 5), SYS_OK);
    EXPECT(sys_stt_check(&valid[5], 16), SYS_OK);

    // ---- designs Section 2.2 rules out
    const sys_stt_design_t invalid[] = {
        design(1, 1, 1, 1, 0, 0, 0, 0, 0, 0, 0, 1),                // singular
        design(1, 0, 1, 0, 0, 0, 0, 0, 0, 0, 0, 1),                // sums read before they exist
        design(1, 1, 0, -1, 1, -1, 1, 0, 0, 0, 0, 1),              // SBM run backwards
        design(1, 0, 0, 1, 1, 1, -1, 0, 0, 0, 0, 1),               // FBS whose inputs come from the future (s.e = -1)
        design(1, 0, 0, 1, 0, 0, 0, 1, 1, 0, 0, 1),                // weights passed within one step
        design(1, 0, 0, 1, 1, -1, 2, 0, 0, 0, 0, 1),               // X dependence changes the input
        design(1, 0, 0, 1, 1, 0, 0, 0, 0, 0, 0, 1),                // null X dependence
        design(1, 0, 1, 1, 0, 0, 0, 1, 1, 1, 0, 1),                // W dependence changes the tap
        design(1, 0, 1, 1, 0, 0, 0, 0, 0, 0, 1, 1),                // Z dependence across outputs
        design(1, 0, 0, 1, 0, 0, 0, 0, 0, 0, 0, 2),                // Z dependence skips taps
    };
    for (const sys_stt_design_t& d : invalid)
        for (int k : {1, 2, 5, 64}) EXPECT(sys_stt_check(&d, k), SYS_ERR_DESIGN);
    // ---- valid, but beyond the kernel
    const sys_stt_design_t too_large[] = {
        design(1, 0, 1, 2, 0, 0, 0, 0, 0, 0, 0, 1),                // |det| = 2
        design(1, 3, 0, 1, 1, -1, 1, 0, 0, 0, 0, 1),               // values jump over PEs
        design(1, 0, 4, 1, 0, 0, 0, 1, 1, 0, 0, 1),                // weights travel four steps
        design(65, 1, 64, 1, 0, 0, 0, 0, 0, 0, 0, 1),              // coefficient beyond +-64
        design(INT_MAX, 1, INT_MIN, 1, 0, 0, 0, 0, 0, 0, 0, 1),    // arithmetic on these must not overflow
        design(INT_MIN, INT_MIN, INT_MAX, INT_MAX, 1, INT_MAX, INT_MIN, 1, INT_MIN, 0, 0, 1),
    };
    for (const sys_stt_design_t& d : too_large)
        for (int k : {1, 5, 64}) {
            const int st = sys_stt_check(&d, k);
            if (st != SYS_ERR_UNSUPPORTED && st != SYS_ERR_DESIGN) {
                fprintf(stderr, "oversized design accepted (%s)\n", sys_status_string(st));
                ++failures;
            }
        }
    EXPECT(sys_stt_check(nullptr, 5), SYS_ERR_NULL);
    EXPECT(sys_stt_check(&valid[0], 0), SYS_ERR_SIZE);
    EXPECT(sys_stt_check(&valid[0], SYS_MAX_K1D + 1), SYS_ERR_SIZE);
    EXPECT(sys_conv1d_stt(X, 100, taps.data(), 5, Y, &invalid[0], nullptr), SYS_ERR_DESIGN);
    EXPECT(sys_conv1d_stt(X, 100, taps.data(), 5, X + 10, &valid[0], nullptr), SYS_ERR_ALIAS);
    EXPECT(sys_conv1d_stt(X, 100, taps.data(), 5, Y, nullptr, nullptr), SYS_ERR_NULL);

    // ---- argument validation of the convolutions: refused before any launch
    EXPECT(sys_conv1d(nullptr, 100, taps.data(), 5, Y, SYS_PROJ_FBS, nullptr), SYS_ERR_NULL);
    EXPECT(sys_conv1d(X, 100, taps.data(), 0, Y, SYS_PROJ_FBS, nullptr), SYS_ERR_SIZE);
    EXPECT(sys_conv1d(X, 4, taps.data(), 5, Y, SYS_PROJ_FBS, nullptr), SYS_ERR_SIZE);
    EXPECT(sys_conv1d(X, 100, taps.data(), 65, Y, SYS_PROJ_FBS, nullptr), SYS_ERR_UNSUPPORTED);
    EXPECT(sys_conv1d(X, 100, taps.data(), 5, Y, SYS_PROJ_MFMA, nullptr), SYS_ERR_UNSUPPORTED);
    EXPECT(sys_conv1d(X, 100, taps.data(), 5, Y, 99, nullptr), SYS_ERR_UNSUPPORTED);
    EXPECT(sys_conv1d((float*)((char*)X + 2), 100, taps.data(), 5, Y, SYS_PROJ_FBS, nullptr), SYS_ERR_UNSUPPORTED);
    EXPECT(sys_conv1d(X, (size_t)1 << 41, taps.data(), 5, Y, SYS_PROJ_FBS, nullptr), SYS_ERR_UNSUPPORTED);
    EXPECT(sys_conv1d(X, 100, taps.data(), 5, X + 99, SYS_PROJ_FBS, nullptr), SYS_ERR_ALIAS);
    EXPECT(sys_conv1d(X, SIZE_MAX / 8, taps.data(), 5, Y, SYS_PROJ_FBS, nullptr), SYS_ERR_UNSUPPORTED);
    EXPECT(sys_conv1d_strided(X, 100, taps.data(), 5, 0, Y, SYS_PROJ_FBS, nullptr), SYS_ERR_SIZE);
    EXPECT(sys_conv1d_strided(X, 100, taps.data(), 5, 3, Y, SYS_PROJ_FBS, nullptr), SYS_ERR_UNSUPPORTED);
    EXPECT(sys_conv1d_strided(X, 100, taps.data(), 5, 2, X + 10, SYS_PROJ_FBS, nullptr), SYS_ERR_ALIAS);
    EXPECT(sys_conv1d_strided(X, 100, taps.data(), 5, INT_MAX, Y, SYS_PROJ_SBM, nullptr), SYS_ERR_UNSUPPORTED);

    EXPECT(sys_conv2d(X, 10, 10, 10, nullptr, 3, 3, Y, 8, SYS_PROJ_FBS, nullptr), SYS_ERR_NULL);
    EXPECT(sys_conv2d(X, 10, 10, 9, taps.data(), 3, 3, Y, 8, SYS_PROJ_FBS, nullptr), SYS_ERR_SIZE);
    EXPECT(sys_conv2d(X, 10, 10, 10, taps.data(), 3, 3, Y, 7, SYS_PROJ_FBS, nullptr), SYS_ERR_SIZE);
    EXPECT(sys_conv2d(X, 10, 10, 10, taps.data(), 11, 3, Y, 8, SYS_PROJ_FBS, nullptr), SYS_ERR_SIZE);
    EXPECT(sys_conv2d(X, 100, 100, 100, taps.data(), 16, 3, Y, 98, SYS_PROJ_FBS, nullptr), SYS_ERR_UNSUPPORTED);
    EXPECT(sys_conv2d(X, 100, 100, 100, taps.data(), 4, 3, Y, 98, SYS_PROJ_BFS, nullptr), SYS_ERR_UNSUPPORTED);
    EXPECT(sys_conv2d(X, 100, 100, 100, taps.data(), 14, 3, Y, 98, SYS_PROJ_MFMA, nullptr), SYS_ERR_UNSUPPORTED);
    EXPECT(sys_conv2d(X, 100, 100, 100, taps.data(), 3, 3, X + 5000, 98, SYS_PROJ_FBS, nullptr), SYS_ERR_ALIAS);
    EXPECT(sys_conv2d(X, 100, 100, (size_t)1 << 32, taps.data(), 3, 3, Y, 98, SYS_PROJ_FBS, nullptr), SYS_ERR_UNSUPPORTED);
    EXPECT(sys_conv2d(X, 1, INT_MAX, (size_t)INT_MAX, taps.data(), 1, 1, (float*)0x7000000000, (size_t)INT_MAX,
                      SYS_PROJ_AUTO, nullptr), SYS_ERR_UNSUPPORTED);
    EXPECT(sys_conv2d(X, INT_MAX, 1, 1, taps.data(), 15, 1, X + 4, 1, SYS_PROJ_AUTO, nullptr), SYS_ERR_ALIAS);
    EXPECT(sys_conv2d_strided(X, 100, 100, 100, taps.data(), 3, 3, 0, Y, 98, SYS_PROJ_FBS, nullptr), SYS_ERR_SIZE);
    EXPECT(sys_conv2d_strided(X, 100, 100, 100, taps.data(), 3, 3, 3, Y, 98, SYS_PROJ_FBS, nullptr), SYS_ERR_UNSUPPORTED);
    EXPECT(sys_conv2d_strided(X, 100, 100, 100, taps.data(), 15, 15, 2, X + 5000, 49, SYS_PROJ_FBS, nullptr), SYS_ERR_ALIAS);

    // ---- the matrix-core projection derives a scale from the taps on the host: every tap is read, none beyond
    for (int kh = 1; kh <= 13; ++kh)
        for (int kw = 1; kw <= 13; ++kw) {
            std::vector<float> f((size_t)kh * kw, 0.0f);           // exactly kh * kw floats on the heap
            EXPECT(sys_conv2d(X, 100, 100, 100, f.data(), kh, kw, X + 5000, 100 - kw + 1, SYS_PROJ_MFMA, nullptr), SYS_ERR_ALIAS);
            f.back() = 1e-33f;
            EXPECT(sys_conv2d(X, 100, 100, 100, f.data(), kh, kw, X + 5000, 100 - kw + 1, SYS_PROJ_MFMA, nullptr), SYS_ERR_UNSUPPORTED);
            f.back() = INFINITY; f.front() = kh * kw > 1 ? 3e33f : INFINITY;
            EXPECT(sys_conv2d(X, 100, 100, 100, f.data(), kh, kw, X + 5000, 100 - kw + 1, SYS_PROJ_MFMA, nullptr),
                   kh * kw > 1 ? SYS_ERR_UNSUPPORTED : SYS_ERR_ALIAS);
            f.front() = NAN; f.back() = -0.5f;
            EXPECT(sys_conv2d(X, 100, 100, 100, f.data(), kh, kw, X + 5000, 100 - kw + 1, SYS_PROJ_MFMA, nullptr), SYS_ERR_ALIAS);
        }

    // ---- queries over their whole domain and beyond
    for (int p = -2; p <= 10; ++p)
        for (int k = -1; k <= 70; ++k) {
            (void)sys_conv1d_has(p, k);
            (void)sys_conv1d_strided_has(p, k, 2);
            for (int kw = -1; kw <= 17; ++kw) { (void)sys_conv2d_has(p, k, kw); (void)sys_conv2d_strided_has(p, k, kw, 2); }
        }
    for (int s = -3; s <= 12; ++s) if (!sys_status_string(s) || !sys_projection_name(s)) ++failures;
    EXPECT(sys_copy_f32(X, X + 1, 10, nullptr), SYS_ERR_ALIAS);
    EXPECT(sys_copy_f32(X, Y, 0, nullptr), SYS_ERR_SIZE);
    EXPECT(sys_last_hip_error(), 0);
    if (sys_version() < 200) ++failures;

    printf(failures ? "FAILED (%d)\n" : "clean\n", failures);
    return failures ? 1 : 0;
}
