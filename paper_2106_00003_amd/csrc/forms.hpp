// Rotation forms of the float carousel kernels: constants and the rule that picks the form of a call
// from the largest |theta| (shared by the coefficient kernels, the sweeps and the host).
#pragma once
#include <hip/hip_runtime.h>

namespace givens {

enum { kFormStandard = 0, kFormScaled = 1, kFormLifted = 2 };

constexpr int kRenormPeriod = 64;                 // blocks between renormalisations of the scaled and lifted forms
constexpr float kScaledMaxAbsTheta = 0.78539816f; // scaled form only when every |theta| <= pi/4
constexpr float kLiftedMaxAbsTheta = 1.0e6f;      // lifted form only when every |theta| is at most this


// Which form a call runs, from the largest |theta| (NaN compares false everywhere: standard form).
// scaled_max is kScaledMaxAbsTheta, or negative when the caller has asked for no scaled form.
__host__ __device__ __forceinline__ int form_for_range(float max_abs, float scaled_max)
{
    if (max_abs <= scaled_max) return kFormScaled;
    if (max_abs <= kLiftedMaxAbsTheta) return kFormLifted;
    return kFormStandard;
}
__device__ __forceinline__ int selected_form(const unsigned *flag, float scaled_max)
{
    if (!flag) return kFormStandard;
    return form_for_range(__uint_as_float(*flag), scaled_max);
}
// true when `form` is the one the flag selects (flag == nullptr: standard form, always)
__device__ __forceinline__ bool form_selected(const unsigned *flag, int form, float scaled_max)
{
    return selected_form(flag, scaled_max) == form;
}

} // namespace givens
