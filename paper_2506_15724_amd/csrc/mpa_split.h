// The Eq. 8 split of one head's candidate total over the modalities (paper Sec. 3.3), in integers:
// used by the allocation kernel (prompt eviction) and by the re-eviction during generation.
#pragma once
#include <hip/hip_runtime.h>

namespace madakv {

// ah tokens over M <= 4 modalities with masses wm (as floats: the values that cross the interface)
// and candidate counts nm; result bm.
//   two modalities   b_t = floor(share_t * ah + 0.5), b_v = ah - b_t; a modality short of candidates
//                    hands the surplus to the other
//   more             quotas share_m * ah floored, spare tokens to the largest fractional parts (ties:
//                    lower id); a modality short of candidates is cut to what it has, the surplus goes to
//                    the others in order of decreasing share (ties: lower id)
//   mpa_mode 0       no split: the total in slot 0;  2 / 3: fixed priority, text / image (ascending /
//                    descending id) takes all it can
// The double arithmetic must round after every operation (a fused multiply-add keeps the exact
// product and changes which of two nearly equal fractional parts is the larger).
__device__ __forceinline__ void mpa_split_device(long long ah, const float (&wm)[4], const long long (&nm)[4], int M, int mpa_mode,
                                                 long long (&bm)[4]) {
#pragma clang fp contract(off)
  constexpr int MAXM = 4;
#pragma unroll
  for (int m = 0; m < MAXM; ++m) bm[m] = 0;
  if (mpa_mode == 0) { bm[0] = ah; return; }
  if (M == 2) {
    const long long n_t = nm[0], n_v = nm[1];
    // the share is formed in double from the float masses
    const double wt = (double)wm[0], wv = (double)wm[1];
    const double tot = wt + wv;
    double share;
    if (tot > 0.0) share = wt / tot;
    else share = (n_t + n_v) > 0 ? (double)n_t / (double)(n_t + n_v) : 0.0;
    if (mpa_mode == 2) share = 1.0;
    else if (mpa_mode == 3) share = 0.0;
    long long bt = (long long)floor(share * (double)ah + 0.5);
    long long bv = ah - bt;
    if (bt > n_t) { bt = n_t; bv = ah - n_t; }
    if (bv > n_v) { bv = n_v; bt = ah - n_v; }
    bm[0] = bt; bm[1] = bv;
    return;
  }
  if (mpa_mode == 2 || mpa_mode == 3) {
    long long left = ah;
    for (int j = 0; j < M; ++j) {
      const int m = mpa_mode == 2 ? j : M - 1 - j;
      bm[m] = left < nm[m] ? left : nm[m];
      left -= bm[m];
    }
    return;
  }
  double tot = 0.0; long long nt = 0;
  for (int m = 0; m < M; ++m) { tot += (double)wm[m]; nt += nm[m]; }
  double share[MAXM] = {0, 0, 0, 0}, frac[MAXM] = {0, 0, 0, 0};
  long long sumb = 0;
  for (int m = 0; m < M; ++m) {
    share[m] = tot > 0.0 ? (double)wm[m] / tot : (nt > 0 ? (double)nm[m] / (double)nt : 0.0);
    const double quota = share[m] * (double)ah;
    bm[m] = (long long)floor(quota);
    frac[m] = quota - (double)bm[m];
    sumb += bm[m];
  }
  const long long spare = ah - sumb;
  long long add[MAXM] = {0, 0, 0, 0};
  for (int m = 0; m < M; ++m) {
    int rank = 0;
    for (int o = 0; o < M; ++o) if (frac[o] > frac[m] || (frac[o] == frac[m] && o < m)) ++rank;
    add[m] = rank < spare ? 1 : 0;
  }
  long long surplus = 0;
  for (int m = 0; m < M; ++m) {
    bm[m] += add[m];
    if (bm[m] > nm[m]) { surplus += bm[m] - nm[m]; bm[m] = nm[m]; }
  }
  for (int r = 0; r < M; ++r) {                 // r-th largest share takes what it has room for
    for (int m = 0; m < M; ++m) {
      int rank = 0;
      for (int o = 0; o < M; ++o) if (share[o] > share[m] || (share[o] == share[m] && o < m)) ++rank;
      if (rank == r) {
        const long long room = nm[m] - bm[m];
        const long long give = surplus < room ? surplus : room;
        bm[m] += give; surplus -= give;
      }
    }
  }
}

}  // namespace madakv
