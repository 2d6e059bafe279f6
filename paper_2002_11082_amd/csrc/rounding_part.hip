// libogq: one object file per bucket capacity of the random-rounding quantize kernels (the instantiations of
// one capacity take about as long to compile as the rest of the library).  OGQ_PART = 1, 2, 4, 8: one
// wavefront per bucket of at most 256 * OGQ_PART elements; 16: two wavefronts per bucket of at most 4096
// elements (measured 6-17 % faster there than one wavefront holding 64 elements per lane; for 2048 elements one
// wavefront is the faster choice); 102: four wavefronts of 2048 elements per bucket of at most 8192 (22-37 % faster
// than two wavefronts of 4096: half the registers, twice the resident wavefronts); 104, 108: 4, 8 wavefronts of 4096
// elements per bucket of at most 16384, 32768 (there eight of 2048 are slower, sixteen mixed).
#include "rounding_kernels.h"

#include "launch.h"

#ifndef OGQ_PART
#error "compile with -DOGQ_PART=<capacity>"
#endif

namespace ogq {

#define OGQ_CAT2(a, b) a##b
#define OGQ_CAT(a, b) OGQ_CAT2(a, b)

#if OGQ_PART == 16
void launch_rounding_c16(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes, hipStream_t st)
{
    launch_orq_team_levels<2, 8>(g, n, p, nb, lv, codes, st);
}
#elif OGQ_PART < 100
void OGQ_CAT(launch_rounding_c, OGQ_PART)(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv,
                                          void* codes, hipStream_t st)
{
    launch_orq_levels<OGQ_PART>(g, n, p, nb, lv, codes, st);
}
#elif OGQ_PART == 102
void launch_rounding_w2(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes, hipStream_t st)
{
    launch_orq_team_levels<4, 8>(g, n, p, nb, lv, codes, st);
}
#elif OGQ_PART == 104
void launch_rounding_w4(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes, hipStream_t st)
{
    launch_orq_team_levels<4, 16>(g, n, p, nb, lv, codes, st);
}
#elif OGQ_PART == 108
void launch_rounding_w8(const float* g, size_t n, const ogq_params_t* p, uint32_t nb, float* lv, void* codes, hipStream_t st)
{
    launch_orq_team_levels<8, 16>(g, n, p, nb, lv, codes, st);
}
#else
#error "unknown OGQ_PART"
#endif

}  // namespace ogq
