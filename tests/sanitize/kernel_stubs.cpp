// Stand-ins for the kernels' launch functions, so that the host-only sources of libpvq link into a CPU program.
// A call to any of them means that the program under test touched the GPU path: it aborts.
#include <cstdio>
#include <cstdlib>

#include "pvq_internal.h"

static hipError_t reached(const char *what)
{
    fprintf(stderr, "kernel launch function %s reached in a host-only program\n", what);
    abort();
}

bool pvq_encode_fits(const pvq_ctx *, const pvq_encode_args &) { return true; }
hipError_t pvq_launch_encode(const pvq_ctx *, const pvq_encode_args &, int, hipStream_t) { return reached("pvq_launch_encode"); }
hipError_t pvq_launch_fill_zero(float *, int64_t, hipStream_t) { return reached("pvq_launch_fill_zero"); }
hipError_t pvq_launch_correct(const pvq_ctx *, float *, int64_t, int64_t, int64_t, const float *, int64_t, float *, hipStream_t) { return reached("pvq_launch_correct"); }
int64_t pvq_correct_static_max_rows(void) { return 8192; }
int64_t pvq_correct_front_tiles(int64_t) { return 1536; }
hipError_t pvq_launch_correct_static(const pvq_ctx *, float *, int64_t, int64_t, int64_t, const float *, int64_t, hipStream_t) { return reached("pvq_launch_correct_static"); }
hipError_t pvq_launch_size_table(int, int, int, uint32_t *, uint32_t *, hipStream_t) { return reached("pvq_launch_size_table"); }
hipError_t pvq_launch_hadamard(const void *, int, int64_t, int64_t, int64_t, int, const uint8_t *, int, void *, int, int64_t, hipStream_t) { return reached("pvq_launch_hadamard"); }
hipError_t pvq_wide_launch_encode(const pvq_ctx *, const pvq_encode_args &, int, hipStream_t) { return reached("pvq_wide_launch_encode"); }
hipError_t pvq_wide_launch_decode(const pvq_ctx *, const pvq_decode_args &, int, hipStream_t) { return reached("pvq_wide_launch_decode"); }
hipError_t pvq_wide_launch_rotate_encode(const pvq_ctx *, const pvq_encode_args &, int, int, const uint8_t *, hipStream_t) { return reached("pvq_wide_launch_rotate_encode"); }
bool pvq_encode8_usable(const pvq_ctx *, const pvq_encode_args &) { return false; }
hipError_t pvq_encode8_launch(const pvq_ctx *, const pvq_encode_args &, int, hipStream_t) { return reached("pvq_encode8_launch"); }
bool pvq_fast8_decode_usable(const pvq_ctx *, const pvq_decode_args &) { return false; }
bool pvq_fast8_gemv_usable(const pvq_ctx *, const pvq_decode_args &) { return false; }
hipError_t pvq_fast8_launch_decode(const pvq_ctx *, const pvq_decode_args &, int, hipStream_t) { return reached("pvq_fast8_launch_decode"); }
hipError_t pvq_fast8_launch_gemv(const pvq_ctx *, const pvq_decode_args &, hipStream_t) { return reached("pvq_fast8_launch_gemv"); }
int pvq_fast8_plan_gemv(const pvq_ctx *, const pvq_decode_args &, pvq_gemv_pass *) { (void)reached("pvq_fast8_plan_gemv"); return 0; }
hipError_t pvq_fast8_prepare(void) { return reached("pvq_fast8_prepare"); }
bool pvq_walk_usable(const pvq_ctx *) { return false; }
hipError_t pvq_walk_launch_decode(const pvq_ctx *, const pvq_decode_args &, int, hipStream_t) { return reached("pvq_walk_launch_decode"); }
hipError_t pvq_walk_launch_gemv(const pvq_ctx *, const pvq_decode_args &, hipStream_t) { return reached("pvq_walk_launch_gemv"); }
bool pvq_rotate_encode8_usable(const pvq_ctx *, const pvq_encode_args &, int) { return false; }
hipError_t pvq_rotate_encode8_launch(const pvq_ctx *, const pvq_encode_args &, int, int, const uint8_t *, hipStream_t) { return reached("pvq_rotate_encode8_launch"); }
