// Adaptive parallelism switching (Sec. 4.3, Eq. 2-3, Alg. 1): host-side controller that turns the
// per-step denoising discrepancy M into the stage boundaries tau1, tau2.  No device work.
//
// Steps are counted upwards in sampling order, i = 0 .. T-1 (the paper's listing counts timesteps
// downwards and indexes the window inconsistently; on an ascending index the slope of Eq. 2 is
// taken as the rate of decline G_i = (M[i-L] - M[i]) / L, which is >= 0 while the curve falls).
// tau1' is the first i >= L with 0 <= G_i < g_slope; tau1 = min(tau1', cap), and tau1 = cap once step
// cap is reached without the test having fired (safety cap); tau2 = tau1 + k (Eq. 3).  Eq. 3 bounds the
// interval by 1 <= k < T - tau1 (tau2 is a step of the run, so a fully-connecting stage exists) and the
// safety cap is an upper bound of tau1, so the cap in force is cap = min(tau_cap, T - 1 - k): the bound
// then holds for every history, also when the run is shorter than tau_cap + k + 1 steps.  k >= T admits
// no tau1 and is rejected.
// Stages: 0 warm-up (i <= tau1), 1 parallelism (tau1 < i < tau2), 2 fully-connecting (i >= tau2).
#include "common.h"

extern "C" int hyb_switch_init(hyb_switch_state* s, int total_steps, int window, float g_slope, int tau_cap, int k) {
    HYB_CHECK_PTR(s);
    HYB_REQUIRE(total_steps > 0 && total_steps <= HYB_SWITCH_MAX_STEPS, HYB_ERR_SHAPE,
                "hyb_switch_init: total_steps %d must be in [1, %d]", total_steps, HYB_SWITCH_MAX_STEPS);
    HYB_REQUIRE(window > 0 && k >= 1 && tau_cap >= 0 && g_slope > 0.f, HYB_ERR_SHAPE,
                "hyb_switch_init: need window > 0, k >= 1, tau_cap >= 0, g_slope > 0");
    HYB_REQUIRE(k <= total_steps - 1, HYB_ERR_SHAPE,
                "hyb_switch_init: k = %d leaves no tau1 >= 0 with k < total_steps - tau1 (Eq. 3), total_steps = %d", k, total_steps);
    s->total_steps = total_steps;
    s->window = window;
    s->g_slope = g_slope;
    s->tau_cap = tau_cap;
    s->k = k;
    s->step = 0;
    s->tau1 = -1;
    s->tau2 = -1;
    for (int i = 0; i < HYB_SWITCH_MAX_STEPS; i++) s->history[i] = 0.0;
    return HYB_OK;
}

extern "C" int hyb_switch_stage(const hyb_switch_state* s, int step) {
    if (s == nullptr || s->tau1 < 0 || step <= s->tau1) return 0;
    return step < s->tau2 ? 1 : 2;
}

extern "C" int hyb_switch_push(hyb_switch_state* s, float discrepancy, int* stage) {
    HYB_CHECK_PTR(s);
    HYB_REQUIRE(s->step < s->total_steps, HYB_ERR_SHAPE, "hyb_switch_push: all %d steps were already pushed", s->total_steps);
    const int i = s->step;
    s->history[i] = (double)discrepancy;
    const int cap = s->tau_cap < s->total_steps - 1 - s->k ? s->tau_cap : s->total_steps - 1 - s->k;   // Eq. 3
    if (s->tau1 < 0) {
        int fire = -1;
        if (i >= s->window) {
            const double g = (s->history[i - s->window] - s->history[i]) / (double)s->window;
            if (g >= 0.0 && g < (double)s->g_slope) fire = i;
        }
        if (fire < 0 && i >= cap) fire = cap;     // safety cap
        if (fire >= 0) {
            s->tau1 = fire < cap ? fire : cap;
            s->tau2 = s->tau1 + s->k;
        }
    }
    s->step = i + 1;
    if (stage) *stage = hyb_switch_stage(s, i);
    return HYB_OK;
}
