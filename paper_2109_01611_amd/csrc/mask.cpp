// CU-mask arithmetic of a gpu-let: percent -> CUs per die -> mask words.
// Pure integer host code (paper Sec. 2.3: a gpu-let holds a fraction of the
// GPU's compute; Sec. 4.3 Split: sizes p and 100-p).
#include "gpulet.h"

namespace {

// Shader engines per die.  CU c of a die sits in shader engine c % kEngines, and the hardware
// deals workgroups round-robin to the engines of a die whatever the mask, so the engine with the
// fewest CUs inside the mask sets the pace: a share that is not a multiple of kEngines runs no
// faster than the next lower multiple (measured on MI355X: 26 CUs per die slower than 24, 13
// slower than 12, 6 as fast as 4).
constexpr int kEngines = 4;

// CUs per die of a which = 0 gpu-let of `pct` percent: the nearest multiple of kEngines (half
// rounds up), kept inside kEngines .. cpx - kEngines for a gpu-let smaller than the whole GPU so
// that its Split partner always exists and is balanced too.  Dies whose CU count is not a
// multiple of kEngines (or too small to split that way) fall back to rounding to whole CUs,
// 1 .. cpx - 1.
int share0(int pct, int cpx) {
    if (pct >= 100) return cpx;
    if (pct <= 0) return 0;
    if (cpx % kEngines == 0 && cpx >= 2 * kEngines) {
        int n = kEngines * ((pct * cpx + 50 * kEngines) / (100 * kEngines));
        if (n > cpx - kEngines) n = cpx - kEngines;
        if (n < kEngines) n = kEngines;
        return n;
    }
    int n = (pct * cpx + 50) / 100;
    if (n > cpx - 1) n = cpx - 1;
    if (n < 1) n = 1;
    return n;
}

}  // namespace

extern "C" gpulet_status gpulet_mask_for_pct(int n_cu_total, int n_xcd, int pct, int which,
                                             uint32_t *words, int n_words_cap, int *n_words,
                                             int *n_cu) {
    if (!words || !n_words || !n_cu) return GPULET_EINVAL;
    if (pct < 1 || pct > 100 || which < 0 || which > 1) return GPULET_EINVAL;
    if (n_xcd < 1 || n_cu_total < 1 || n_cu_total % n_xcd != 0) return GPULET_EINVAL;
    const int cpx = n_cu_total / n_xcd;
    int lo, hi;  // CU indices [lo, hi) taken in every die
    if (which == 0) {
        lo = 0;
        hi = share0(pct, cpx);
    } else {
        lo = share0(100 - pct, cpx);
        hi = cpx;
    }
    if (hi - lo < 1) return GPULET_EINVAL;
    const int nw = (n_cu_total + 31) / 32;
    if (n_words_cap < nw) return GPULET_ENOMEM;
    for (int i = 0; i < nw; ++i) words[i] = 0u;
    // Bit i of the mask is CU (i / n_xcd) of die (i % n_xcd).
    for (int bit = lo * n_xcd; bit < hi * n_xcd; ++bit) words[bit >> 5] |= 1u << (bit & 31);
    *n_words = nw;
    *n_cu = (hi - lo) * n_xcd;
    return GPULET_OK;
}

extern "C" const char *gpulet_status_string(gpulet_status s) {
    switch (s) {
        case GPULET_OK: return "GPULET_OK";
        case GPULET_EINVAL: return "GPULET_EINVAL: invalid argument";
        case GPULET_EOVERSUB: return "GPULET_EOVERSUB: gpu-lets on this device would exceed two or 100%";
        case GPULET_EHIP: return "GPULET_EHIP: HIP runtime error";
        case GPULET_ENOMEM: return "GPULET_ENOMEM: workspace or output array too small";
        default: return "GPULET_E?: unknown status";
    }
}
