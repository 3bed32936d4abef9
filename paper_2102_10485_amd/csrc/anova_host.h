// Host part of the one-way analysis of variance (Section 4 of the paper: the F-statistic per channel): from the
// per-label sums, counts and within-label squared deviations that the device kernels leave, the ratio of the
// between-label to the within-label mean square.  Shared by the two entry points that run those kernels.
#pragma once

namespace gan {

// gsum, ssw: [K][C]; gcnt: [K].  Returns false (and leaves F at 0) when fewer than two labels occur or there are not
// more images than labels.
inline bool anova_f_from_sums(const double* gsum, const double* ssw, const int* gcnt, int K, int C, double* F) {
  for (int ch = 0; ch < C; ++ch) F[ch] = 0.0;
  int kk = 0;
  long long nn = 0;
  for (int k = 0; k < K; ++k) { kk += gcnt[k] > 0; nn += gcnt[k]; }
  if (kk < 2 || nn <= kk) return false;
  for (int ch = 0; ch < C; ++ch) {
    double all = 0.0;
    for (int k = 0; k < K; ++k) all += gsum[(long long)k * C + ch];
    const double grand = all / (double)nn;
    double ssb = 0.0, sw = 0.0;
    for (int k = 0; k < K; ++k) {
      if (gcnt[k] == 0) continue;
      const double mk = gsum[(long long)k * C + ch] / (double)gcnt[k];
      ssb += (double)gcnt[k] * (mk - grand) * (mk - grand);
      sw += ssw[(long long)k * C + ch];
    }
    F[ch] = (ssb / (double)(kk - 1)) / (sw / (double)(nn - kk));
  }
  return true;
}

}  // namespace gan
